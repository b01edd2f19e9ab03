"""GPU parity of the sparse wire format (this library's own format for the same packed words; the paper
defines none): the encoder against the oracle's statement of the format, bit for bit on every defined
word; decode-and-sum and the fused step on sparse streams against the oracle's dense results, bit for
bit -- the method itself is untouched by the format."""
import numpy as np
import pytest
import torch

from helpers import assert_bits_equal

pytestmark = pytest.mark.gpu

SIZES = [1, 15, 16, 17, 63, 64, 65, 1023, 4095, 4096, 4097, 4111, 8191, 8192, 8193, 12289, 65536, 100003]


@pytest.fixture(scope="module")
def B():
    from paper_2106_10796_amd import binding, build
    build.ensure_built()
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def _words(rng, n, density):
    nw = (n + 15) // 16
    w = rng.integers(1, 1 << 32, nw, dtype=np.uint64).astype(np.uint32)
    w[rng.random(nw) >= density] = 0
    return w


@pytest.mark.parametrize("density", [0.0, 1.0, 0.03, 0.5])
@pytest.mark.parametrize("n", SIZES)
def test_sparse_encode(B, oracle, n, density):
    rng = np.random.default_rng(8000 + n)
    word = _words(rng, n, density)
    want, want_seg = oracle.sparse_encode(word, n, fill=0x5A5A5A5A)
    GUARD = 16
    full = torch.full((B.sparse_words(n) + 2 * GUARD,), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    sparse = full[GUARD: GUARD + B.sparse_words(n)]
    seg = torch.full((B.sparse_segments(n),), -1, dtype=torch.int32, device="cuda")
    assert B.sparse_words(n) == want.size and B.sparse_segments(n) == want_seg.size
    dpacked = torch.from_numpy(word.view(np.int32)).cuda()
    B.cdsgd_sparse_encode(dpacked, n, sparse, seg)
    torch.cuda.synchronize()
    # slots the format leaves alone keep the sentinel on both sides, so the whole buffer must match
    assert_bits_equal(sparse.cpu().numpy(), want.view(np.int32), "sparse n=%d density=%g" % (n, density))
    assert_bits_equal(seg.cpu().numpy(), want_seg.view(np.int32), "segment_words n=%d" % n)
    f = full.cpu().numpy()
    assert (f[:GUARD] == 0x5A5A5A5A).all() and (f[GUARD + want.size:] == 0x5A5A5A5A).all()
    assert_bits_equal(dpacked.cpu().numpy(), word.view(np.int32), "packed must not be written")
    B.cdsgd_sparse_encode(dpacked, n, sparse, None)      # the per-segment counts are optional
    torch.cuda.synchronize()
    assert_bits_equal(sparse.cpu().numpy(), want.view(np.int32), "sparse, no counts")


@pytest.mark.parametrize("t", [0.5, 0.05])
@pytest.mark.parametrize("N", [1, 3, 4, 5, 16, 17, 64])
def test_decode_sum_sparse(B, oracle, N, t):
    rng = np.random.default_rng(8100 + N)
    for n in (1, 17, 4095, 4097, 20000):
        # real quantiser output of differing densities, plus the unused code 3 in one worker
        words = []
        for j in range(N):
            g = rng.normal(0, t * (0.2 + 0.25 * (j % 5)), n).astype(np.float32)
            words.append(oracle.quantize_pack(g, np.zeros(n, np.float32), t))
        words[0][::3] |= np.uint32(3)
        if n % 16:
            for w in words:
                w[-1] &= np.uint32((1 << (2 * (n % 16))) - 1)
        sparse = [torch.from_numpy(oracle.sparse_encode(w, n, fill=0x7F7F7F7F)[0].view(np.int32)).cuda() for w in words]
        agg = torch.full((n + 8,), 9.0, device="cuda")
        B.cdsgd_decode_sum_sparse(sparse, agg[:n], t)
        torch.cuda.synchronize()
        want = oracle.decode_sum(words, n, t)
        assert_bits_equal(agg[:n].cpu().numpy(), want, "agg N=%d n=%d t=%g" % (N, n, t))
        assert bool((agg[n:] == 9.0).all())


def _run_sparse_layer_list(B, oracle, sizes, N, self_rank, k, t, steps, seed, grad_std):
    rng = np.random.default_rng(seed)
    T = len(sizes)
    dev = dict(device="cuda")
    W0 = [rng.normal(0, 0.3, n).astype(np.float32) for n in sizes]
    st = dict(w_global=[torch.from_numpy(w).cuda() for w in W0],
              w_local=[torch.zeros(n, **dev) for n in sizes],
              residual=[torch.zeros(n, **dev) for n in sizes],
              grad=[torch.zeros(n, **dev) for n in sizes],
              packed_self=[torch.full((B.packed_words(n),), -1, dtype=torch.int32, **dev) for n in sizes],
              agg_full=[torch.zeros(n, **dev) for n in sizes])
    peers = [None if j == self_rank else [torch.full((B.sparse_words(n),), 0x33333333, dtype=torch.int32, **dev)
                                          for n in sizes] for j in range(N)]
    plan = B.Plan([{key: st[key][i] for key in st} for i in range(T)], peers if N > 1 else None, N, self_rank,
                  peers_sparse=True)
    sims = [oracle.Simulation(W0[i], N, k, t, 0.4, 0.1, self_rank) for i in range(T)]
    sent_words = total_words = 0
    for s in range(steps):
        outs = []
        for i, n in enumerate(sizes):
            grads = [rng.normal(0, grad_std, n).astype(np.float32) for _ in range(N)]
            comp, agg, words = sims[i].step(grads)
            outs.append((comp, words))
            st["grad"][i].copy_(torch.from_numpy(grads[self_rank]))
            if comp:
                for j in range(N):
                    if j != self_rank:
                        sp, seg = oracle.sparse_encode(words[j], n, fill=0x33333333)
                        peers[j][i].copy_(torch.from_numpy(sp.view(np.int32)))
                        sent_words += int(seg.sum())
                        total_words += words[j].size
            else:
                st["agg_full"][i].copy_(torch.from_numpy(agg))
        plan.step(s, k, t, 0.4, 0.1)
        torch.cuda.synchronize()
        for i, n in enumerate(sizes):
            comp, words = outs[i]
            tag = "step %d tensor %d (n=%d)" % (s, i, n)
            if comp:
                assert_bits_equal(st["packed_self"][i].cpu().numpy(), words[self_rank].view(np.int32), "packed " + tag)
            assert_bits_equal(st["residual"][i].cpu().numpy(), sims[i].residual[self_rank], "residual " + tag)
            assert_bits_equal(st["w_global"][i].cpu().numpy(), sims[i].w_global, "w_global " + tag)
            assert_bits_equal(st["w_local"][i].cpu().numpy(), sims[i].w_local, "w_local " + tag)
    plan.destroy()
    return sent_words, total_words


RAGGED = [1, 10, 16, 17, 64, 100, 1000, 4095, 4096, 4097, 9000, 36864, 5, 20011]


@pytest.mark.parametrize("t", [0.5, 0.05])
@pytest.mark.parametrize("N,self_rank", [(1, 0), (2, 1), (4, 0), (5, 2), (9, 8), (10, 0), (16, 9), (17, 16), (64, 31)])
def test_fused_step_with_sparse_peers(B, oracle, N, self_rank, t):
    """Dense-ish codes (gradient std = 1.1 t: a third of the codes fire, almost every word non-zero)."""
    _run_sparse_layer_list(B, oracle, RAGGED, N, self_rank, k=3, t=t, steps=4, seed=8200 + 17 * N + self_rank,
                           grad_std=1.1 * t)


def test_fused_step_with_sparse_peers_when_little_is_sent(B, oracle):
    """Small gradients: most words are zero, a few fire as the residuals build up; the wire carries far
    fewer words than the packed form."""
    sent, total = _run_sparse_layer_list(B, oracle, RAGGED + [3 * 4096 + 7], 8, 3, k=4, t=0.5, steps=7, seed=8300,
                                         grad_std=0.11)
    assert 0 < sent < 0.5 * total
    sent, total = _run_sparse_layer_list(B, oracle, [4096 * 3 + 50], 16, 0, k=4, t=0.5, steps=3, seed=8301,
                                         grad_std=0.005)
    assert sent == 8 * 15 * 2 * 4        # nothing fires: bitmaps only (4 segments, 15 peers, 2 compressed steps)


def test_sparse_argument_errors(B):
    from paper_2106_10796_amd.binding import ERR_PARAM
    n = 100
    mk = lambda: torch.zeros(n, device="cuda")
    t = dict(w_global=mk(), w_local=mk(), residual=mk(), grad=mk(), packed_self=B.new_packed(n))
    plan = B.Plan([t], [None, [B.new_sparse(n)]], 2, 0, peers_sparse=True)
    with pytest.raises(B.CdsgdError) as e:
        plan.set_peer_format(2)
    assert e.value.status == ERR_PARAM
    plan.set_peer_format(B.PEERS_PACKED)
    plan.destroy()
