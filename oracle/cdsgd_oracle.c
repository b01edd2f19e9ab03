/*
 * CD-SGD hot-path oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, scalar CPU statement of what one iteration of CD-SGD's
 * formal-training loop computes on the data-parallel path: 2-bit threshold
 * quantisation with an error-feedback residual, packing of the codes,
 * decode-and-sum over N workers, and the two weight updates.  It exists so
 * that the HIP library can be checked against something written directly from
 * the paper.  It shares no code with the HIP path, is never called by it, and
 * may be imported only by tests, the smoke check and the benchmark's
 * cpu-baseline leg.
 *
 * One element at a time, one worker at a time, fp32 with round-to-nearest-even
 * (the paper trains in fp32), no blocking, no SIMD intrinsics, no reordering.
 * Build: gcc -O2 -fno-fast-math -ffp-contract=off (so that no multiply-add is
 * fused behind our back and denormals are kept).
 *
 * Where each function comes from:
 *   oracle_quantize      Sec. 2.3 (residual buffer of BIT-SGD) and Sec. 3.4.1
 *                        (values beyond the threshold are sent as the threshold,
 *                        the error is kept and re-offered later)
 *   oracle_pack/unpack   Sec. 3.2.2 (32-bit gradients encoded into 2 bits and
 *                        written to sml_buf); the bit layout is this build's
 *                        convention, the paper gives none
 *   oracle_decode_sum    Sec. 3.2.1 (server decodes to 32 bits before updating)
 *                        and the sum in eq. 10
 *   oracle_full_sum      the sum in eq. 1 / Alg. 1 correction branch
 *   oracle_update        eq. 10 (global) and eq. 11 (local)
 *   oracle_step          Alg. 1, FormalTraining, one pass of the while loop
 *   oracle_warmup_step   Alg. 1, WARMUP, one pass of the while loop
 *   oracle_trainer_step  Alg. 1 as a whole: WARMUP for i = 0..n, then FormalTraining
 *   oracle_cost_model    eq. 2, 4, 5, 6, 7 (iteration times); the savings are the
 *                        differences T_loc - T_cd and T_bit - T_cd that Sec. 3.3 defines
 *   oracle_sparse_encode/decode   no passage: a wire format of this build for the same
 *                        packed words (Sec. 7 only names sparsification as future work)
 *
 * Every function here is pinned by tests/test_oracle_pins.py (hand-unrolled
 * recurrence, closed forms, invariants, brute force on tiny inputs).  The
 * points that are readings of a silent paper (boundary case |a| == t, the code
 * values and word layout, the initial counter value, the residual on correction
 * iterations, and the two hand-over readings stated at oracle_warmup_step and
 * oracle_trainer_step: what the local buffer holds when WARMUP has n == 0, and
 * the base of the first FormalTraining local update) are pinned only to this
 * build's stated reading; for the last two that reading is eq. 11.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

/* 2-bit code values (this build's convention; 3 is never produced). */
#define ORACLE_CODE_ZERO 0u
#define ORACLE_CODE_POS 1u
#define ORACLE_CODE_NEG 2u

/* Value a 2-bit code stands for (Sec. 3.4.1: the sent value equals the
 * threshold in magnitude).  The unused code 3 decodes to zero. */
float oracle_dequant(uint8_t code, float t)
{
    if (code == ORACLE_CODE_POS) return t;
    if (code == ORACLE_CODE_NEG) return -t;
    return 0.0f;
}

/* Error-feedback threshold quantiser for one worker (Sec. 2.3, Sec. 3.4.1).
 * a = r + g is what is offered; if it has reached the threshold the threshold
 * is sent and the rest stays in the residual, otherwise nothing is sent and
 * everything stays.  residual is updated in place, code[e] receives 0/1/2. */
void oracle_quantize(const float *grad, float *residual, uint8_t *code, size_t n, float t)
{
    for (size_t e = 0; e < n; ++e) {
        float a = residual[e] + grad[e];
        if (a >= t) {
            code[e] = ORACLE_CODE_POS;
            residual[e] = a - t;
        } else if (a <= -t) {
            code[e] = ORACLE_CODE_NEG;
            residual[e] = a + t;
        } else {
            code[e] = ORACLE_CODE_ZERO;
            residual[e] = a;
        }
    }
}

/* 16 codes per 32-bit word, element e in bits [2(e%16)+1 : 2(e%16)] of word
 * e/16; unused high bits of the last word are zero (Sec. 3.2.2, sml_buf). */
void oracle_pack(const uint8_t *code, size_t n, uint32_t *word)
{
    size_t nw = (n + 15) / 16;
    for (size_t w = 0; w < nw; ++w) word[w] = 0u;
    for (size_t e = 0; e < n; ++e)
        word[e / 16] |= ((uint32_t)(code[e] & 3u)) << (2 * (e % 16));
}

void oracle_unpack(const uint32_t *word, size_t n, uint8_t *code)
{
    for (size_t e = 0; e < n; ++e)
        code[e] = (uint8_t)((word[e / 16] >> (2 * (e % 16))) & 3u);
}

/* Server side of a compressed iteration: decode every worker's codes back to
 * 32 bits and add them up, workers in index order, starting from +0
 * (Sec. 3.2.1; the sum of eq. 10). */
void oracle_decode_sum(const uint32_t *const *word, int num_workers, float *agg, size_t n, float t)
{
    for (size_t e = 0; e < n; ++e) {
        float s = 0.0f;
        for (int j = 0; j < num_workers; ++j) {
            uint8_t c = (uint8_t)((word[j][e / 16] >> (2 * (e % 16))) & 3u);
            s = s + oracle_dequant(c, t);
        }
        agg[e] = s;
    }
}

/* Server side of a correction iteration: the sum of the workers' 32-bit
 * gradients, same order (eq. 1; Alg. 1, else-branch). */
void oracle_full_sum(const float *const *grad, int num_workers, float *agg, size_t n)
{
    for (size_t e = 0; e < n; ++e) {
        float s = 0.0f;
        for (int j = 0; j < num_workers; ++j) s = s + grad[j][e];
        agg[e] = s;
    }
}

/* eq. 11 then eq. 10, both starting from the same global weight W_k:
 *   Wloc = W - lr_local * g_local          (immediate, 32-bit local gradient)
 *   W    = W - (lr_global / N) * agg       (delayed, aggregated gradient)
 * Each is one fused multiply-add; the scale is rounded to fp32 once.
 * w_local/grad_local may both be NULL (global rule only); agg may be NULL
 * (local rule only). */
void oracle_update(float *w_global, float *w_local, const float *grad_local, const float *agg,
                   size_t n, float lr_local, float lr_global, int num_workers)
{
    float scale = lr_global / (float)num_workers;
    for (size_t e = 0; e < n; ++e) {
        float w = w_global[e];
        if (w_local && grad_local) w_local[e] = fmaf(-lr_local, grad_local[e], w);
        if (agg) w_global[e] = fmaf(-scale, agg[e], w);
    }
}

/* One pass of Alg. 1's FormalTraining loop with FP/BP replaced by given
 * gradients.  count is the loop's counter before the pass.
 *   count % k != 0 : every worker quantises (own residual) and packs; the
 *                    aggregate is the decoded sum.
 *   count % k == 0 : correction iteration, no quantisation, residuals and
 *                    packed buffers are left alone; the aggregate is the sum of
 *                    the 32-bit gradients.
 * The observed worker `self` updates its local weights from the pre-step global
 * weights with its own 32-bit gradient in both cases.
 * residual[j], grad[j], word[j] are per-worker arrays; code_scratch has n bytes.
 * Returns 1 for a compressed iteration, 0 for a correction iteration. */
int oracle_step(float *w_global, float *w_local, float *const *residual, const float *const *grad,
                uint32_t *const *word, float *agg, uint8_t *code_scratch, size_t n, int num_workers,
                int self, long count, int k, float t, float lr_local, float lr_global)
{
    int compressed = (count % k) != 0;
    if (compressed) {
        for (int j = 0; j < num_workers; ++j) {
            oracle_quantize(grad[j], residual[j], code_scratch, n, t);
            oracle_pack(code_scratch, n, word[j]);
        }
        oracle_decode_sum((const uint32_t *const *)word, num_workers, agg, n, t);
    } else {
        oracle_full_sum(grad, num_workers, agg, n);
    }
    oracle_update(w_global, w_local, grad[self], agg, n, lr_local, lr_global, num_workers);
    return compressed;
}

/* One pass of Alg. 1's WARMUP loop (Sec. 3.2.1) with FP/BP replaced by given
 * gradients; i is the loop counter before the pass, n the number of warm-up
 * steps (the loop runs for i = 0..n).  Every pass is plain S-SGD on the global
 * weights (eq. 1): the server sums the workers' 32-bit gradients and updates.
 *   i == n     : the local buffer, which holds the global weights W_n of this
 *                pass, is first updated in place with the own gradient (eq. 11
 *                with k = n: W_loc = W_n - lr_local * g_n)
 *   i == n - 1 : after the pull, the new global weights W_n are copied into the
 *                local buffer
 * Reading for n == 0: the algorithm has no pass n - 1 in which to make that copy,
 * so nothing it states ever loads the local buffer.  Eq. 11 and eq. 3 fix what
 * the buffer must hold when it is updated -- the global weights of the pass
 * (Sec. 3.1: the local buffer loads the global weights of the last iteration
 * as local weights) -- so for n == 0 the copy is made at the start of pass 0,
 * from the initial global weights.  Whatever the caller left in the local
 * buffer is never read.
 * No quantisation happens, residuals are not touched. */
void oracle_warmup_step(float *w_global, float *w_local, const float *const *grad, float *agg, size_t n_elems,
                        int num_workers, int self, long i, long n, float lr_local, float lr_global)
{
    oracle_full_sum(grad, num_workers, agg, n_elems);
    if (i == n) {
        if (n == 0) memcpy(w_local, w_global, n_elems * sizeof(float)); /* the copy no earlier pass could make */
        /* the local buffer holds W_n here and is updated in place */
        for (size_t e = 0; e < n_elems; ++e) w_local[e] = fmaf(-lr_local, grad[self][e], w_local[e]);
    }
    oracle_update(w_global, NULL, NULL, agg, n_elems, lr_local, lr_global, num_workers);
    if (i == n - 1) memcpy(w_local, w_global, n_elems * sizeof(float));
}

/* Alg. 1 end to end for iteration number `iter` (0, 1, 2, ...): iterations
 * 0..n are WARMUP passes, iteration n+1+c is FormalTraining's pass with
 * count = c.  Returns 0 for a warm-up pass, 1 for a compressed pass, 2 for a
 * correction pass.
 * Reading for the hand-over: every FormalTraining pass, the first included,
 * takes the base of its local update from the global weights as they stand
 * before the pass (eq. 11: W_loc = W_k - lr_local * g).  In later passes that
 * is what Alg. 1's copy after the pull left in the local buffer; WARMUP's last
 * pass has no such copy, so read as buffer contents alone the first formal
 * pass would start from W_n - lr_local * g_n instead of W_{n+1}.  Eq. 11 decides. */
int oracle_trainer_step(float *w_global, float *w_local, float *const *residual, const float *const *grad,
                        uint32_t *const *word, float *agg, uint8_t *code_scratch, size_t n_elems,
                        int num_workers, int self, long iter, long warmup_n, int k, float t, float lr_local,
                        float lr_global)
{
    if (iter <= warmup_n) {
        oracle_warmup_step(w_global, w_local, grad, agg, n_elems, num_workers, self, iter, warmup_n, lr_local,
                           lr_global);
        return 0;
    }
    return oracle_step(w_global, w_local, residual, grad, word, agg, code_scratch, n_elems, num_workers, self,
                       iter - warmup_n - 1, k, t, lr_local, lr_global)
               ? 1
               : 2;
}

/* Sparse form of a packed stream -- THIS BUILD'S OWN FORMAT, not the paper's: Sec. 7 names a
 * combination with sparsification as future work and defines nothing, so these two functions
 * follow the definition in the library's header and are pinned only to that definition (a
 * hand-worked fixture, round trips on every tail, densities 0 and 1).  The method itself is
 * untouched: a decoded sparse stream is the packed stream again, word for word.
 *
 * A stream of nw = ceil(n / 16) words is cut into segments of 256 words (4096 elements).
 * Segment s occupies words [264 s, 264 s + 264) of the sparse buffer: first 8 bitmap words
 * (bit b of bitmap word m set iff packed word 256 s + 32 m + b exists and is non-zero), then
 * the non-zero words of the segment in index order; the slots after them are left as they are.
 * seg_words[s] receives 8 + (number of non-zero words): what a sender would put on the wire. */
void oracle_sparse_encode(const uint32_t *word, size_t n, uint32_t *sparse, uint32_t *seg_words)
{
    size_t nw = (n + 15) / 16;
    size_t nseg = (nw + 255) / 256;
    for (size_t s = 0; s < nseg; ++s) {
        uint32_t *seg = sparse + 264 * s;
        uint32_t count = 0;
        for (int m = 0; m < 8; ++m) seg[m] = 0u;
        for (size_t i = 0; i < 256; ++i) {
            size_t w = 256 * s + i;
            if (w < nw && word[w] != 0u) {
                seg[i / 32] |= 1u << (i % 32);
                seg[8 + count] = word[w];
                ++count;
            }
        }
        if (seg_words) seg_words[s] = 8u + count;
    }
}

/* Inverse of oracle_sparse_encode: rebuilds the nw packed words. */
void oracle_sparse_decode(const uint32_t *sparse, size_t n, uint32_t *word)
{
    size_t nw = (n + 15) / 16;
    for (size_t w = 0; w < nw; ++w) {
        const uint32_t *seg = sparse + 264 * (w / 256);
        size_t i = w % 256;
        if ((seg[i / 32] >> (i % 32)) & 1u) {
            uint32_t before = 0; /* set bits below bit i of the segment's bitmap */
            for (size_t b = 0; b < i; ++b) before += (seg[b / 32] >> (b % 32)) & 1u;
            word[w] = seg[8 + before];
        } else {
            word[w] = 0u;
        }
    }
}

/* The paper's time model, from the definitions only (in double: these are
 * modelled times, not fp32 training state).  out[0..6] = T_ssgd (eq. 2), T_loc
 * (eq. 4), T_bit (eq. 5), phi_cd (eq. 6), T_cd (eq. 7), T_loc - T_cd, T_bit - T_cd
 * (the two savings as Sec. 3.3 defines them, not the case tables of eq. 8/9). */
void oracle_cost_model(double tau, double phi, double psi, double delta, int k, long i, double *out)
{
    double t_ssgd = tau + phi;
    double t_loc = tau > phi ? tau : phi;
    double t_bit = tau + delta + psi;
    double phi_cd = (i % k != 0) ? delta + psi : phi;
    double t_cd = tau > phi_cd ? tau : phi_cd;
    out[0] = t_ssgd;
    out[1] = t_loc;
    out[2] = t_bit;
    out[3] = phi_cd;
    out[4] = t_cd;
    out[5] = t_loc - t_cd;
    out[6] = t_bit - t_cd;
}
