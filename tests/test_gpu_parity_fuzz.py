"""Seeded random configurations of Alg. 1 end to end through cdsgd_trainer_step: layer lists,
worker counts and positions, periods, warm-up lengths, thresholds (one per call or one per
tensor, both decode forms), gradient types (fp32, bf16, fp16), both sources of the 32-bit
aggregate, peers' streams packed or in the sparse form, bounded grids -- every iteration
compared with the oracle's trainer bit for bit.
CDSGD_FUZZ_CASES raises the number of cases for a longer soak; CDSGD_FUZZ_SEED moves the stream."""
import os

import numpy as np
import pytest
import torch

from helpers import assert_bits_equal

pytestmark = pytest.mark.gpu

TORCH_OF = {"float32": torch.float32, "bfloat16": torch.bfloat16, "float16": torch.float16}


@pytest.fixture(scope="module")
def B():
    from paper_2106_10796_amd import binding, build
    build.ensure_built()
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def _round_to(g, dtype_name):
    """The fp32 values a 16-bit gradient buffer will hold (rounded once, here, by torch on the CPU)."""
    if dtype_name == "float32":
        return g
    return torch.from_numpy(g).to(TORCH_OF[dtype_name]).float().numpy()


def draw_case(rng):
    T = int(rng.integers(1, 9))
    sizes = []
    for kind in rng.integers(0, 4, T):
        if kind == 0:
            sizes.append(int(rng.integers(1, 70)))                                      # tiny, every tail shape
        elif kind == 1:
            sizes.append(int(rng.integers(1, 5)) * 4096 + int(rng.integers(-3, 4)))     # around chunk edges
        elif kind == 2:
            sizes.append(int(rng.integers(70, 20000)))
        else:
            sizes.append(int(rng.integers(1, 40)) * 1024)
    N = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 31, 33]))
    pool = [0.5, 0.25, 2.0, 0.05, 0.3, 1e-3, 0.0625, 7.0]
    per_tensor = bool(rng.integers(0, 3) == 0)
    if per_tensor:
        # all powers of two (count form) or a mix (chain form for every tensor)
        src = [0.5, 0.25, 2.0, 0.0625] if rng.integers(0, 2) else pool
        thresholds = [float(rng.choice(src)) for _ in range(T)]
    else:
        thresholds = None
    return dict(sizes=sizes, N=N, self_rank=int(rng.integers(0, N)), k=int(rng.integers(1, 5)),
                warmup_n=int(rng.integers(0, 4)), t=float(rng.choice(pool)), thresholds=thresholds,
                dtype=str(rng.choice(["float32", "float32", "bfloat16", "float16"])),
                full_grads=bool(rng.integers(0, 2)), formal=int(rng.integers(2, 7)),
                sparse_peers=bool(rng.integers(0, 3) == 0), max_workgroups=int(rng.choice([0, 0, 0, 1, 3, 50])))


def run_case(B, oracle, c, seed):
    rng = np.random.default_rng(seed)
    sizes, N, self_rank, k, warmup_n = c["sizes"], c["N"], c["self_rank"], c["k"], c["warmup_n"]
    T = len(sizes)
    th = c["thresholds"] or [c["t"]] * T
    gd = TORCH_OF[c["dtype"]]
    lr_l, lr_g = 0.4, 0.1
    dev = dict(device="cuda")
    W0 = [rng.normal(0, 0.3, n).astype(np.float32) for n in sizes]
    st = dict(w_global=[torch.from_numpy(w).cuda() for w in W0],
              w_local=[torch.full((n,), -5.5, **dev) for n in sizes],
              residual=[torch.zeros(n, **dev) for n in sizes],
              grad=[torch.zeros(n, dtype=gd, **dev) for n in sizes],
              packed_self=[torch.full((B.packed_words(n),), -1, dtype=torch.int32, **dev) for n in sizes],
              agg_full=[torch.zeros(n, **dev) for n in sizes])
    sparse = c["sparse_peers"]
    peers = [None if j == self_rank else [(B.new_sparse(n) if sparse else B.new_packed(n)) for n in sizes]
             for j in range(N)]
    peer_g = [None if j == self_rank else [torch.zeros(n, dtype=gd, **dev) for n in sizes] for j in range(N)]
    plan = B.Plan([{key: st[key][i] for key in st} for i in range(T)], peers if N > 1 else None, N, self_rank,
                  grad_dtype=gd, peers_sparse=sparse)
    plan.set_max_workgroups(c["max_workgroups"])
    if c["full_grads"]:
        plan.bind_full_grads(peer_g)
    if c["thresholds"]:
        plan.set_thresholds(th)
    trainer = B.Trainer(plan, warmup_n, k, c["t"], lr_l, lr_g)
    sims = [oracle.TrainerSimulation(W0[i], N, warmup_n, k, th[i], lr_l, lr_g, self_rank,
                                     w_local0=np.full(sizes[i], -5.5, np.float32)) for i in range(T)]
    for it in range(warmup_n + 1 + c["formal"]):
        outs = []
        for i, n in enumerate(sizes):
            grads = [_round_to(rng.normal(0, 1.1 * th[i], n).astype(np.float32), c["dtype"]) for _ in range(N)]
            mode, agg, words = sims[i].step(grads)
            outs.append((mode, words))
            st["grad"][i].copy_(torch.from_numpy(grads[self_rank]).to(gd))
            for j in range(N):
                if j == self_rank:
                    continue
                if mode == 1:
                    wire = oracle.sparse_encode(words[j], n, fill=0x11111111)[0] if sparse else words[j]
                    peers[j][i].copy_(torch.from_numpy(wire.view(np.int32)))
                elif c["full_grads"]:
                    peer_g[j][i].copy_(torch.from_numpy(grads[j]).to(gd))
            if mode != 1 and not c["full_grads"]:
                st["agg_full"][i].copy_(torch.from_numpy(agg))
        res_before = [r.clone() for r in st["residual"]]
        kind = trainer.step()
        torch.cuda.synchronize()
        for i, n in enumerate(sizes):
            mode, words = outs[i]
            assert mode == kind
            tag = "iteration %d (mode %d) tensor %d (n=%d, t=%g)" % (it, mode, i, n, th[i])
            if mode == 1:
                assert_bits_equal(st["packed_self"][i].cpu().numpy(), words[self_rank].view(np.int32), "packed " + tag)
            else:
                assert torch.equal(st["residual"][i], res_before[i]), "residual touched " + tag
            assert_bits_equal(st["residual"][i].cpu().numpy(), sims[i].residual[self_rank], "residual " + tag)
            assert_bits_equal(st["w_global"][i].cpu().numpy(), sims[i].w_global, "w_global " + tag)
            if it >= warmup_n - 1:
                assert_bits_equal(st["w_local"][i].cpu().numpy(), sims[i].w_local, "w_local " + tag)
            else:
                assert bool((st["w_local"][i] == -5.5).all()), "w_local written early " + tag
    trainer.destroy()
    plan.destroy()


def test_random_trainer_configurations(B, oracle):
    cases = int(os.environ.get("CDSGD_FUZZ_CASES", "30"))
    seed0 = int(os.environ.get("CDSGD_FUZZ_SEED", "20261128"))
    rng = np.random.default_rng(seed0)
    seen = set()
    for case in range(cases):
        c = draw_case(rng)
        seen.add((c["dtype"], c["full_grads"], c["thresholds"] is not None, c["warmup_n"] == 0))
        try:
            run_case(B, oracle, c, seed0 + 1 + case)
        except AssertionError as e:
            raise AssertionError("case %d %r: %s" % (case, c, e))
        if cases > 100 and case % 100 == 99:
            print("fuzz: %d cases done" % (case + 1), flush=True)
    assert len(seen) >= min(cases, 30) // 3      # the draw really varies type, aggregate source, thresholds
