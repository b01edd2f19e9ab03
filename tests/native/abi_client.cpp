// A client of the C ABI that knows nothing of Python or torch: device memory from hipMalloc, a
// layer list stepped through Alg. 1 with cdsgd_trainer_* (warm-up, then formal training with
// k-step correction; full gradients bound, so the 32-bit passes sum in the kernel), and every
// buffer compared bit for bit, after every iteration, with the CPU oracle's trainer.  A second
// pass steps the formal phase layer by layer with cdsgd_step_fused_range and on a stream of
// its own.  Test code: it links the oracle, which the library never does.
//
// Usage: abi_client [seed]     exit status 0 and a last line "abi client ok ..." on success.
#include <hip/hip_runtime_api.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "cdsgd.h"

extern "C" {
// the oracle's trainer (oracle/cdsgd_oracle.c)
int oracle_trainer_step(float *w_global, float *w_local, float *const *residual, const float *const *grad,
                        uint32_t *const *word, float *agg, uint8_t *code_scratch, size_t n_elems, int num_workers,
                        int self, long iter, long warmup_n, int k, float t, float lr_local, float lr_global);
}

namespace {

#define HIP_OK(call)                                                                                    \
    do {                                                                                                \
        hipError_t e_ = (call);                                                                         \
        if (e_ != hipSuccess) {                                                                         \
            std::printf("%s:%d: %s -> %s\n", __FILE__, __LINE__, #call, hipGetErrorString(e_));         \
            std::exit(2);                                                                               \
        }                                                                                               \
    } while (0)

#define LIB_OK(call)                                                                                    \
    do {                                                                                                \
        int s_ = (call);                                                                                \
        if (s_ != CDSGD_OK) {                                                                           \
            std::printf("%s:%d: %s -> %d (%s)\n", __FILE__, __LINE__, #call, s_, cdsgd_status_string(s_)); \
            std::exit(3);                                                                               \
        }                                                                                               \
    } while (0)

// Inputs only: a 64-bit mixing counter generator and a triangular distribution scaled to the
// threshold, so that about a third of the elements fire.  None of the method's arithmetic.
struct Rng {
    uint64_t s;
    uint32_t next()
    {
        s += 0x9E3779B97F4A7C15ull;
        uint64_t z = s;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return (uint32_t)((z ^ (z >> 31)) >> 32);
    }
    float unit() { return (float)(next() >> 8) * (1.0f / 16777216.0f); }  // [0, 1)
    float value(float scale) { return (unit() + unit() - 1.0f) * scale; }
};

template <class T>
T *dev_alloc(size_t count)
{
    void *p = nullptr;
    HIP_OK(hipMalloc(&p, count * sizeof(T) + 16));
    return static_cast<T *>(p);
}

struct Layer {
    size_t n = 0, words = 0;
    float *w_global = nullptr, *w_local = nullptr, *residual = nullptr, *grad = nullptr;
    uint32_t *packed_self = nullptr;
    std::vector<uint32_t *> peer_packed;  // [worker], null at self
    std::vector<float *> peer_grad;       // [worker], null at self
    // the oracle's copy of every worker's state
    std::vector<float> o_wg, o_wl, o_agg;
    std::vector<std::vector<float>> o_res, o_grad;
    std::vector<std::vector<uint32_t>> o_word;
    std::vector<uint8_t> o_code;
};

int compare_bits(const char *what, const void *dev, const void *host, size_t bytes, int layer, long iter)
{
    std::vector<unsigned char> got(bytes);
    HIP_OK(hipMemcpy(got.data(), dev, bytes, hipMemcpyDeviceToHost));
    if (std::memcmp(got.data(), host, bytes) == 0) return 0;
    size_t at = 0;
    while (got[at] == static_cast<const unsigned char *>(host)[at]) ++at;
    std::printf("MISMATCH %s: layer %d iteration %ld, first differing byte %zu of %zu\n", what, layer, iter, at, bytes);
    return 1;
}

int run(uint64_t seed, int N, int self, long warmup_n, int k, float t, bool by_ranges)
{
    const size_t sizes[] = {1, 17, 4097, 9000, 36864, 70001};
    const int T = (int)(sizeof(sizes) / sizeof(sizes[0]));
    const float lr_local = 0.4f, lr_global = 0.1f;
    Rng rng{seed};
    hipStream_t stream = nullptr;
    if (by_ranges) HIP_OK(hipStreamCreateWithFlags(&stream, hipStreamNonBlocking));

    std::vector<Layer> layers((size_t)T);
    std::vector<cdsgd_tensor> desc((size_t)T);
    for (int i = 0; i < T; ++i) {
        Layer &L = layers[(size_t)i];
        L.n = sizes[i];
        L.words = cdsgd_packed_words(L.n);
        L.w_global = dev_alloc<float>(L.n);
        L.w_local = dev_alloc<float>(L.n);
        L.residual = dev_alloc<float>(L.n);
        L.grad = dev_alloc<float>(L.n);
        L.packed_self = dev_alloc<uint32_t>(L.words);
        L.peer_packed.assign((size_t)N, nullptr);
        L.peer_grad.assign((size_t)N, nullptr);
        for (int j = 0; j < N; ++j) {
            if (j == self) continue;
            L.peer_packed[(size_t)j] = dev_alloc<uint32_t>(L.words);
            L.peer_grad[(size_t)j] = dev_alloc<float>(L.n);
        }
        L.o_wg.resize(L.n);
        for (float &v : L.o_wg) v = rng.value(0.5f);
        L.o_wl.assign(L.n, -7.0f);  // never read before Alg. 1 writes it
        L.o_agg.assign(L.n, 0.0f);
        L.o_res.assign((size_t)N, std::vector<float>(L.n, 0.0f));
        L.o_grad.assign((size_t)N, std::vector<float>(L.n, 0.0f));
        L.o_word.assign((size_t)N, std::vector<uint32_t>(L.words, 0u));
        L.o_code.assign(L.n, 0);
        HIP_OK(hipMemcpy(L.w_global, L.o_wg.data(), L.n * 4, hipMemcpyHostToDevice));
        HIP_OK(hipMemcpy(L.w_local, L.o_wl.data(), L.n * 4, hipMemcpyHostToDevice));
        HIP_OK(hipMemset(L.residual, 0, L.n * 4));
        HIP_OK(hipMemset(L.packed_self, 0xFF, L.words * 4));
        cdsgd_tensor &d = desc[(size_t)i];
        d.w_global = L.w_global;
        d.w_local = L.w_local;
        d.residual = L.residual;
        d.grad = L.grad;
        d.packed_self = L.packed_self;
        d.agg_full = nullptr;  // the 32-bit passes sum the bound gradients in the kernel
        d.n = L.n;
    }
    // peers[j][i] and peer_grads[j][i]
    std::vector<std::vector<const uint32_t *>> prow((size_t)N, std::vector<const uint32_t *>((size_t)T, nullptr));
    std::vector<std::vector<const float *>> grow((size_t)N, std::vector<const float *>((size_t)T, nullptr));
    std::vector<const uint32_t *const *> peers((size_t)N, nullptr);
    std::vector<const float *const *> peer_grads((size_t)N, nullptr);
    for (int j = 0; j < N; ++j) {
        if (j == self) continue;
        for (int i = 0; i < T; ++i) {
            prow[(size_t)j][(size_t)i] = layers[(size_t)i].peer_packed[(size_t)j];
            grow[(size_t)j][(size_t)i] = layers[(size_t)i].peer_grad[(size_t)j];
        }
        peers[(size_t)j] = prow[(size_t)j].data();
        peer_grads[(size_t)j] = grow[(size_t)j].data();
    }
    cdsgd_plan *plan = nullptr;
    LIB_OK(cdsgd_plan_create(desc.data(), T, N > 1 ? peers.data() : nullptr, N, self, &plan));
    LIB_OK(cdsgd_plan_bind_full_grads(plan, N > 1 ? peer_grads.data() : nullptr));
    cdsgd_trainer *trainer = nullptr;
    LIB_OK(cdsgd_trainer_create(plan, warmup_n, k, t, lr_local, lr_global, &trainer));

    int bad = 0;
    const long iterations = warmup_n + 1 + 2L * k + 1;
    for (long it = 0; it < iterations && !bad; ++it) {
        // inputs of the iteration, and the oracle's pass
        std::vector<int> kind((size_t)T, 0);
        for (int i = 0; i < T; ++i) {
            Layer &L = layers[(size_t)i];
            std::vector<float *> res((size_t)N);
            std::vector<const float *> grd((size_t)N);
            std::vector<uint32_t *> wrd((size_t)N);
            for (int j = 0; j < N; ++j) {
                for (float &v : L.o_grad[(size_t)j]) v = rng.value(2.2f * t);
                res[(size_t)j] = L.o_res[(size_t)j].data();
                grd[(size_t)j] = L.o_grad[(size_t)j].data();
                wrd[(size_t)j] = L.o_word[(size_t)j].data();
            }
            kind[(size_t)i] = oracle_trainer_step(L.o_wg.data(), L.o_wl.data(), res.data(), grd.data(), wrd.data(),
                                                  L.o_agg.data(), L.o_code.data(), L.n, N, self, it, warmup_n, k, t,
                                                  lr_local, lr_global);
            HIP_OK(hipMemcpy(L.grad, L.o_grad[(size_t)self].data(), L.n * 4, hipMemcpyHostToDevice));
            for (int j = 0; j < N; ++j) {
                if (j == self) continue;
                if (kind[(size_t)i] == CDSGD_PASS_COMPRESSED)
                    HIP_OK(hipMemcpy(L.peer_packed[(size_t)j], L.o_word[(size_t)j].data(), L.words * 4,
                                     hipMemcpyHostToDevice));
                else
                    HIP_OK(hipMemcpy(L.peer_grad[(size_t)j], L.o_grad[(size_t)j].data(), L.n * 4,
                                     hipMemcpyHostToDevice));
            }
        }
        // the library's pass
        int pass = -1;
        if (by_ranges && it > warmup_n) {
            // formal phase enqueued layer by layer, last layers first, in three groups
            const long count = it - warmup_n - 1;
            LIB_OK(cdsgd_step_fused_range(plan, 4, 2, count, k, t, lr_local, lr_global, stream));
            LIB_OK(cdsgd_step_fused_range(plan, 1, 3, count, k, t, lr_local, lr_global, stream));
            LIB_OK(cdsgd_step_fused_range(plan, 0, 1, count, k, t, lr_local, lr_global, stream));
            pass = count % k != 0 ? CDSGD_PASS_COMPRESSED : CDSGD_PASS_CORRECTION;
        } else {
            LIB_OK(cdsgd_trainer_step(trainer, stream, &pass));
        }
        HIP_OK(hipStreamSynchronize(stream));
        for (int i = 0; i < T && !bad; ++i) {
            Layer &L = layers[(size_t)i];
            if (pass != kind[(size_t)i]) {
                std::printf("MISMATCH pass kind: library %d, oracle %d (iteration %ld)\n", pass, kind[(size_t)i], it);
                bad = 1;
                break;
            }
            bad |= compare_bits("w_global", L.w_global, L.o_wg.data(), L.n * 4, i, it);
            if (it >= warmup_n - 1) bad |= compare_bits("w_local", L.w_local, L.o_wl.data(), L.n * 4, i, it);
            bad |= compare_bits("residual", L.residual, L.o_res[(size_t)self].data(), L.n * 4, i, it);
            if (pass == CDSGD_PASS_COMPRESSED)
                bad |= compare_bits("packed_self", L.packed_self, L.o_word[(size_t)self].data(), L.words * 4, i, it);
        }
    }
    LIB_OK(cdsgd_trainer_destroy(trainer));
    LIB_OK(cdsgd_plan_destroy(plan));
    for (Layer &L : layers) {
        HIP_OK(hipFree(L.w_global));
        HIP_OK(hipFree(L.w_local));
        HIP_OK(hipFree(L.residual));
        HIP_OK(hipFree(L.grad));
        HIP_OK(hipFree(L.packed_self));
        for (uint32_t *p : L.peer_packed)
            if (p) HIP_OK(hipFree(p));
        for (float *p : L.peer_grad)
            if (p) HIP_OK(hipFree(p));
    }
    if (stream) HIP_OK(hipStreamDestroy(stream));
    std::printf("case N=%d self=%d warmup=%ld k=%d t=%g %s: %s (%ld iterations)\n", N, self, warmup_n, k, (double)t,
                by_ranges ? "formal phase by ranges on its own stream" : "trainer on the null stream",
                bad ? "FAILED" : "bit-exact", iterations);
    std::fflush(stdout);
    return bad;
}

}  // namespace

int main(int argc, char **argv)
{
    const uint64_t seed = argc > 1 ? std::strtoull(argv[1], nullptr, 10) : 2106;
    int count = 0;
    HIP_OK(hipGetDeviceCount(&count));
    if (count < 1) {
        std::printf("no GPU\n");
        return 2;
    }
    HIP_OK(hipSetDevice(0));
    std::printf("library build %s\n", cdsgd_build_id());
    int bad = 0;
    bad |= run(seed + 1, 4, 1, 2, 3, 0.25f, false);   // count form of the decode, one-wave pieces
    bad |= run(seed + 2, 16, 15, 0, 4, 0.3f, false);  // chain form, four-wave pieces, no warm-up pass before the copy
    bad |= run(seed + 3, 1, 0, 1, 2, 0.5f, false);    // a single worker
    bad |= run(seed + 4, 9, 4, 1, 3, 0.05f, true);    // ranges, own stream
    if (bad) {
        std::printf("abi client FAILED\n");
        return 1;
    }
    std::printf("abi client ok: 4 cases bit-exact against the oracle\n");
    return 0;
}
