/* Drives every oracle function on exactly-sized heap buffers with ragged sizes, for a
 * build with -fsanitize=address,undefined: any out-of-bounds access, signed overflow or
 * bad shift in the oracle aborts the run.  Prints a checksum so that the work cannot be
 * optimised away. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

float oracle_dequant(uint8_t code, float t);
void oracle_quantize(const float *grad, float *residual, uint8_t *code, size_t n, float t);
void oracle_pack(const uint8_t *code, size_t n, uint32_t *word);
void oracle_unpack(const uint32_t *word, size_t n, uint8_t *code);
void oracle_decode_sum(const uint32_t *const *word, int num_workers, float *agg, size_t n, float t);
void oracle_full_sum(const float *const *grad, int num_workers, float *agg, size_t n);
void oracle_update(float *w_global, float *w_local, const float *grad_local, const float *agg, size_t n,
                   float lr_local, float lr_global, int num_workers);
int oracle_trainer_step(float *w_global, float *w_local, float *const *residual, const float *const *grad,
                        uint32_t *const *word, float *agg, uint8_t *code_scratch, size_t n_elems,
                        int num_workers, int self, long iter, long warmup_n, int k, float t, float lr_local,
                        float lr_global);
void oracle_cost_model(double tau, double phi, double psi, double delta, int k, long i, double *out);
void oracle_sparse_encode(const uint32_t *word, size_t n, uint32_t *sparse, uint32_t *seg_words);
void oracle_sparse_decode(const uint32_t *sparse, size_t n, uint32_t *word);

static uint32_t rng_state = 12345u;
static float rnd(void)
{
    rng_state = rng_state * 1664525u + 1013904223u;
    return ((float)(rng_state >> 8) / 8388608.0f) - 1.0f; /* [-1, 1) */
}

int main(void)
{
    double check = 0.0;
    const size_t sizes[] = {1, 2, 15, 16, 17, 31, 33, 100, 1000};
    enum { N = 5 };
    for (size_t si = 0; si < sizeof(sizes) / sizeof(sizes[0]); ++si) {
        size_t n = sizes[si], nw = (n + 15) / 16;
        float *W = malloc(n * sizeof(float)), *L = malloc(n * sizeof(float)), *agg = malloc(n * sizeof(float));
        uint8_t *code = malloc(n);
        float *res[N], *g[N];
        uint32_t *word[N];
        for (int j = 0; j < N; ++j) {
            res[j] = calloc(n, sizeof(float));
            g[j] = malloc(n * sizeof(float));
            word[j] = malloc(nw * sizeof(uint32_t));
        }
        for (size_t e = 0; e < n; ++e) W[e] = L[e] = rnd();
        for (long it = 0; it < 9; ++it) {
            for (int j = 0; j < N; ++j)
                for (size_t e = 0; e < n; ++e) g[j][e] = 0.7f * rnd();
            int mode = oracle_trainer_step(W, L, res, (const float *const *)g, word, agg, code, n, N, (int)(it % N), it, 2,
                                           3, 0.5f, 0.25f, 0.125f);
            check += mode;
        }
        oracle_quantize(g[0], res[0], code, n, 0.05f);
        oracle_pack(code, n, word[0]);
        oracle_unpack(word[0], n, code);
        oracle_decode_sum((const uint32_t *const *)word, N, agg, n, 0.05f);
        oracle_full_sum((const float *const *)g, N, agg, n);
        oracle_update(W, NULL, NULL, agg, n, 0.1f, 0.1f, N);
        oracle_update(W, L, g[1], NULL, n, 0.1f, 0.1f, N);
        for (size_t e = 0; e < n; ++e) check += W[e] + L[e] + agg[e] + code[e];
        for (int j = 0; j < N; ++j) {
            free(res[j]);
            free(g[j]);
            free(word[j]);
        }
        free(W);
        free(L);
        free(agg);
        free(code);
    }
    /* sparse form on exactly-sized buffers: sizes around the 256-word segment edge, sparse and dense words */
    const size_t ssizes[] = {1, 16, 17, 4095, 4096, 4097, 8192, 8200, 3 * 4096 + 5};
    for (size_t si = 0; si < sizeof(ssizes) / sizeof(ssizes[0]); ++si) {
        size_t n = ssizes[si], nw = (n + 15) / 16, nseg = (nw + 255) / 256;
        uint32_t *word = malloc(nw * sizeof(uint32_t)), *back = malloc(nw * sizeof(uint32_t));
        uint32_t *sparse = malloc(nseg * 264 * sizeof(uint32_t)), *seg = malloc(nseg * sizeof(uint32_t));
        for (int dense = 0; dense < 2; ++dense) {
            for (size_t w = 0; w < nw; ++w) word[w] = (dense || rnd() > 0.8f) ? (rng_state | 1u) : 0u;
            for (size_t x = 0; x < nseg * 264; ++x) sparse[x] = 0xA5A5A5A5u;
            oracle_sparse_encode(word, n, sparse, seg);
            oracle_sparse_encode(word, n, sparse, NULL);
            oracle_sparse_decode(sparse, n, back);
            for (size_t w = 0; w < nw; ++w) check += (back[w] == word[w]) ? 0.0 : 1e9;
            for (size_t x = 0; x < nseg; ++x) check += seg[x];
        }
        free(word);
        free(back);
        free(sparse);
        free(seg);
    }
    double out[7];
    for (long i = 0; i < 12; ++i) {
        oracle_cost_model(1.0, 5.0, 1.0, 0.5, 4, i, out);
        check += out[4];
    }
    check += oracle_dequant(3, 0.5f) + oracle_dequant(1, 0.5f);
    printf("oracle driver ok, checksum %.6f\n", check);
    return 0;
}
