/*
 * cdsgd.h -- C ABI of the CD-SGD per-step data-parallel hot path on one GPU.
 *
 * What is computed (arxiv 2106.10796): in every iteration of the formal
 * training phase (Alg. 1) a worker
 *   - updates its local weights at once with its own 32-bit gradient (eq. 11),
 *   - on compressed iterations (count % k != 0) quantises residual + gradient
 *     against a threshold into 2-bit codes, keeping the error in the residual
 *     buffer (Sec. 2.3, Sec. 3.4.1), and writes the codes 16 to a 32-bit word
 *     (Sec. 3.2.2, sml_buf),
 *   - and the global weights are updated with the sum over all N workers of the
 *     decoded codes (Sec. 3.2.1; eq. 10), or, on correction iterations
 *     (count % k == 0), with the sum of the 32-bit gradients (Sec. 3.1).
 *
 * Conventions common to every call
 *   memory     All data pointers are DEVICE pointers owned by the caller unless
 *              a parameter says "host".  The library never frees or keeps them,
 *              except that a plan keeps (borrows) the pointers it was built from.
 *   alignment  fp32 buffers must be 16-byte aligned, packed buffers 4-byte
 *              aligned (CDSGD_ERR_ALIGN otherwise).
 *   aliasing   Within one call or one tensor of a layer list, an output buffer
 *              (residual, w_global, w_local, packed_self, packed, agg) must not overlap
 *              an input or another output, the peers' streams of that tensor included:
 *              CDSGD_ERR_ALIAS.  Buffers of different tensors are not cross-checked.
 *   stream     hip_stream is a hipStream_t passed as void* (NULL = the null
 *              stream).  Work is enqueued and the call returns; nothing
 *              synchronises.
 *   errors     The return value is a cdsgd_status.  Arguments are checked on the
 *              host before any HIP call; on an error nothing has been enqueued.
 *   layout     A packed stream of n elements has cdsgd_packed_words(n) words.
 *              Element e is the 2-bit field at bits [2(e%16)+1 : 2(e%16)] of
 *              word e/16: 00 nothing sent, 01 +threshold, 10 -threshold; 11 is
 *              never written and reads as nothing sent.  Unused bits of the last
 *              word are written as 0.
 *   numbers    fp32, round to nearest even, denormals kept.  Sums over workers
 *              run in worker order 0..N-1 starting from +0.  Each weight update
 *              is one fused multiply-add; lr_global / num_workers is rounded to
 *              fp32 once.  Results do not depend on the launch shape.
 */
#ifndef CDSGD_H
#define CDSGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CDSGD_OK = 0,
    CDSGD_ERR_NULL = 1,    /* a required pointer is NULL */
    CDSGD_ERR_SIZE = 2,    /* n == 0, num_tensors < 1, or a size too large for the launch */
    CDSGD_ERR_PARAM = 3,   /* threshold not finite or <= 0, k < 1, step < 0, rate not finite, bad warm-up index */
    CDSGD_ERR_ALIGN = 4,   /* pointer alignment (see above) */
    CDSGD_ERR_WORKERS = 5, /* num_workers < 1 or > CDSGD_MAX_WORKERS, self out of range */
    CDSGD_ERR_DEVICE = 6,  /* a HIP call failed (allocation, copy, launch) */
    CDSGD_ERR_ALIAS = 7    /* buffers that must be distinct overlap (an output with an input or
                              with another output of the same tensor) */
} cdsgd_status;

#define CDSGD_MAX_WORKERS 64

/* Number of 32-bit words of a packed stream of n elements: ceil(n / 16). */
size_t cdsgd_packed_words(size_t n);

/* Static, NUL-terminated description of a status code. */
const char *cdsgd_status_string(int status);

/* Static, NUL-terminated identity (16 hex digits) of the sources, headers and compiler flags
 * this library was built from, as computed by the build script; lets a harness tell a stale
 * library from a current one.  Not part of the method. */
const char *cdsgd_build_id(void);

/*
 * Quantise and pack one worker's gradient (Sec. 2.3, Sec. 3.4.1, Sec. 3.2.2).
 * Per element: a = residual + grad; a >= t sends +t and keeps a - t; a <= -t
 * sends -t and keeps a + t; otherwise nothing is sent and a is kept.
 *   grad      in   fp32[n]
 *   residual  i/o  fp32[n], updated in place; must not alias grad
 *   packed    out  uint32[cdsgd_packed_words(n)], fully overwritten
 */
int cdsgd_quantize_pack(const float *grad, float *residual, uint32_t *packed, size_t n,
                        float threshold, void *hip_stream);

/*
 * Decode N workers' packed streams to 32 bits and add them up in worker order
 * (Sec. 3.2.1; the sum of eq. 10).
 *   packed  in   HOST array of num_workers DEVICE pointers, each to
 *                uint32[cdsgd_packed_words(n)]; read during the call only
 *   agg     out  fp32[n]
 */
int cdsgd_decode_sum(const uint32_t *const *packed, int num_workers, float *agg, size_t n,
                     float threshold, void *hip_stream);

/*
 * The two update rules, both from the same pre-call global weight (eq. 10, 11):
 *   w_local[e]  = fma(-lr_local, grad_local[e], w_global[e])
 *   w_global[e] = fma(-(lr_global / num_workers), agg[e], w_global[e])
 *   w_global    i/o  fp32[n]
 *   w_local     out  fp32[n]; must not alias w_global
 *   grad_local  in   fp32[n]; w_local and grad_local may both be NULL: global rule only
 *   agg         in   fp32[n]; may be NULL: local rule only, w_global is left alone
 */
int cdsgd_update(float *w_global, float *w_local, const float *grad_local, const float *agg,
                 size_t n, float lr_local, float lr_global, int num_workers, void *hip_stream);

/*
 * Fused step over a layer list (Alg. 1, FormalTraining, one pass): one kernel
 * launch covers every tensor, and each gradient, residual and weight element
 * crosses HBM once.
 *
 * One entry per tensor.  packed_self receives this worker's codes on compressed
 * steps (what would be pushed).  agg_full is the fp32 sum over all N workers of
 * this tensor's 32-bit gradients, read on correction steps only; it may be NULL
 * if the plan is never used for a correction step.
 */
typedef struct {
    float *w_global;        /* i/o fp32[n] */
    float *w_local;         /* out fp32[n] */
    float *residual;        /* i/o fp32[n] (compressed steps) */
    const float *grad;      /* in  fp32[n] this worker's gradient */
    uint32_t *packed_self;  /* out uint32[cdsgd_packed_words(n)] (compressed steps) */
    const float *agg_full;  /* in  fp32[n] (correction steps) or NULL */
    size_t n;
} cdsgd_tensor;

typedef struct cdsgd_plan cdsgd_plan;

/*
 * Build a plan: copies the layer list, the peers' pointers and a chunk table to
 * the device (one small allocation, one synchronous copy; only this call and
 * cdsgd_plan_bind_full_grads allocate).  The plan borrows every data pointer:
 * the buffers must stay alive and in place while the plan is used.
 *   tensors      host array [num_tensors]
 *   peers        host array [num_workers] of host arrays [num_tensors] of device
 *                pointers: peers[j][i] is worker j's packed stream for tensor i
 *                (what would be pulled from the server side).  Row `self` is
 *                ignored and may be NULL: this worker's codes never leave
 *                registers before they are summed.  peers may be NULL when
 *                num_workers == 1.
 *   self         this worker's position in the sum order, 0 <= self < num_workers
 *   out          receives the plan
 */
int cdsgd_plan_create(const cdsgd_tensor *tensors, int num_tensors,
                      const uint32_t *const *const *peers, int num_workers, int self,
                      cdsgd_plan **out);

/* Frees the plan's device tables.  NULL is accepted. */
int cdsgd_plan_destroy(cdsgd_plan *plan);

/*
 * One pass of Alg. 1's loop for every tensor of the plan, `step` being the
 * loop's counter before the pass (it starts at 0).
 *   step % k != 0  compressed: quantise + pack own gradient (residual and
 *                  packed_self written), decode and sum the N streams with the
 *                  own codes at position `self`, then both update rules.
 *   step % k == 0  correction: no quantisation, residual and packed_self are not
 *                  touched; both update rules with the fp32 sum of all gradients as
 *                  the aggregate: summed in the kernel if full gradients are bound
 *                  (cdsgd_plan_bind_full_grads), else read from agg_full
 *                  (CDSGD_ERR_NULL if the plan has neither).
 */
int cdsgd_step_fused(cdsgd_plan *plan, long step, int k, float threshold, float lr_local,
                     float lr_global, void *hip_stream);

/*
 * cdsgd_plan_create for gradients in half the bytes (beyond the paper, which trains in
 * fp32): every pass of the plan reads cdsgd_tensor.grad, and the peers' gradients bound
 * with cdsgd_plan_bind_full_grads, as bf16 or fp16 instead of fp32 (cast the pointers;
 * 16-byte alignment as before).  Each value is widened exactly to fp32 on load;
 * residual, weights, aggregate and every rule stay fp32, so the result is what the fp32
 * path gives on the widened values.  A compressed pass then moves 22 + N/4 bytes per
 * element.  grad_dtype is a cdsgd_grad_dtype (anything else: CDSGD_ERR_PARAM).
 */
typedef enum { CDSGD_GRAD_F32 = 0, CDSGD_GRAD_BF16 = 1, CDSGD_GRAD_F16 = 2 } cdsgd_grad_dtype;
int cdsgd_plan_create_typed(const cdsgd_tensor *tensors, int num_tensors,
                            const uint32_t *const *const *peers, int num_workers, int self,
                            int grad_dtype, cdsgd_plan **out);

/*
 * One threshold per tensor (beyond the paper's single threshold; Sec. 2.3 observes that
 * the parameters of a model differ too much for one value to suit them all).
 *   thresholds  host array [num_tensors], each finite and > 0: compressed passes use
 *               thresholds[i] for tensor i and ignore the threshold argument of the
 *               step call (which is still validated).  NULL goes back to the call's
 *               threshold for every tensor.
 * Rewrites the plan's descriptor table on the device with a synchronous copy: do not
 * call it while a pass of this plan may still be running.
 */
int cdsgd_plan_set_thresholds(cdsgd_plan *plan, const float *thresholds);

/*
 * Split form of cdsgd_step_fused, for overlapping the next forward pass with the
 * rest of the step (Sec. 3.2.2: once the local weights are updated the next
 * iteration can start, whatever quantisation and communication still have to do).
 *   cdsgd_step_local   eq. 11 only, for every tensor: w_local = W - lr_local * grad.
 *                      Reads w_global and grad, writes w_local.
 *   cdsgd_step_global  everything else of the same pass (quantise + pack, decode and
 *                      sum, eq. 10; or the correction branch): same arguments and
 *                      errors as cdsgd_step_fused without lr_local; w_local is not
 *                      touched.  It overwrites w_global, which cdsgd_step_local reads:
 *                      the caller must order it after the cdsgd_step_local of the same
 *                      pass (same stream, or an event).
 * Run in that order the two calls leave exactly what cdsgd_step_fused leaves, at
 * the price of reading grad and w_global twice (36 + N/4 instead of 24 + N/4 bytes
 * per element on a compressed pass).
 */
int cdsgd_step_local(cdsgd_plan *plan, float lr_local, void *hip_stream);
int cdsgd_step_global(cdsgd_plan *plan, long step, int k, float threshold, float lr_global,
                      void *hip_stream);

/*
 * Layer-by-layer form of the three passes above (Sec. 3.2.2: quantisation and communication
 * proceed layer by layer, a layer's turn coming when back-propagation has produced its
 * gradient): the same pass over tensors [first_tensor, first_tensor + num_tensors) of the
 * plan's layer list only.  Nothing of any other tensor is read or written.  Every tensor of the
 * list stepped exactly once with the same `step`, in any order and any grouping, leaves bit for
 * bit what the whole-list call leaves.  The caller keeps `step` the same for all ranges of one
 * iteration; the peers' streams (or agg_full, or the bound gradients) of a range must be in place
 * when its call is enqueued.
 *   errors      those of the whole-list call; CDSGD_ERR_PARAM for first_tensor < 0,
 *               num_tensors < 1 or a range that passes the end of the list.
 */
int cdsgd_step_fused_range(cdsgd_plan *plan, int first_tensor, int num_tensors, long step, int k,
                           float threshold, float lr_local, float lr_global, void *hip_stream);
int cdsgd_step_local_range(cdsgd_plan *plan, int first_tensor, int num_tensors, float lr_local,
                           void *hip_stream);
int cdsgd_step_global_range(cdsgd_plan *plan, int first_tensor, int num_tensors, long step, int k,
                            float threshold, float lr_global, void *hip_stream);

/*
 * Sparse form of a packed stream: a wire format of THIS LIBRARY, not of the paper, which names a
 * combination with sparsification as future work (Sec. 7) and defines nothing; Sec. 2.3 observes
 * that residuals stay below the threshold for long stretches, i.e. that most packed words are zero.
 * The method is untouched: a sparse stream decodes to the packed stream word for word, so every
 * aggregate and weight is bit-identical to the packed path.
 *
 * Format.  The cdsgd_packed_words(n) words of a stream are cut into segments of 256 words (4096
 * elements); there are cdsgd_sparse_segments(n) = ceil(words / 256) of them.  Segment s occupies
 * words [264 s, 264 s + 264) of the sparse buffer (cdsgd_sparse_words(n) = 264 x segments words in
 * all): first 8 bitmap words -- bit b of bitmap word m is set iff packed word 256 s + 32 m + b
 * exists and is non-zero -- then the non-zero packed words of the segment in index order.  The
 * slots behind them are neither written nor read.  A sender puts the first
 * segment_words[s] = 8 + (non-zero words) words of each segment on the wire.
 *
 *   cdsgd_sparse_encode      packed          in   uint32[cdsgd_packed_words(n)]
 *                            sparse          out  uint32[cdsgd_sparse_words(n)]
 *                            segment_words   out  uint32[cdsgd_sparse_segments(n)], may be NULL
 *   cdsgd_decode_sum_sparse  cdsgd_decode_sum (Sec. 3.2.1; the sum of eq. 10) on streams in the
 *                            sparse form: `sparse` is a HOST array of num_workers DEVICE pointers
 *                            to uint32[cdsgd_sparse_words(n)]; same result, bit for bit, as
 *                            cdsgd_decode_sum on the packed streams.
 *   cdsgd_plan_set_peer_format   CDSGD_PEERS_SPARSE: the plan's peers[j][i] pointers are read as
 *                            sparse buffers (cdsgd_sparse_words(n_i) words each) by compressed
 *                            passes; CDSGD_PEERS_PACKED (the default) goes back.  packed_self is
 *                            always written in the packed form.  Host-side setting; anything else
 *                            is CDSGD_ERR_PARAM.  (The overlap checks of cdsgd_plan_create cover
 *                            the packed extent of a peer's buffer only.)
 * A compressed pass then reads 32 bytes + 4 bytes per non-zero word of each peer and chunk instead
 * of 1024 bytes: 24.4 instead of 28 bytes per element at N = 16 when nothing is sent.
 */
typedef enum { CDSGD_PEERS_PACKED = 0, CDSGD_PEERS_SPARSE = 1 } cdsgd_peer_format;
size_t cdsgd_sparse_segments(size_t n);
size_t cdsgd_sparse_words(size_t n);
int cdsgd_sparse_encode(const uint32_t *packed, size_t n, uint32_t *sparse, uint32_t *segment_words,
                        void *hip_stream);
int cdsgd_decode_sum_sparse(const uint32_t *const *sparse, int num_workers, float *agg, size_t n,
                            float threshold, void *hip_stream);
int cdsgd_plan_set_peer_format(cdsgd_plan *plan, int format);

/*
 * Bound the number of workgroups that the passes of this plan launch (Sec. 3.2.2: the rest of
 * the step should not stand in the way of the next iteration's computation).  By default a
 * pass launches one workgroup per 4096-element chunk of the layer list and fills the GPU; with
 * a limit it launches at most max_workgroups workgroups, each walking several chunks, so that
 * a pass enqueued on a second stream leaves compute units to kernels that run beside it.  The
 * results are bit for bit the same for every limit.  0 removes the limit; negative values are
 * CDSGD_ERR_PARAM.  Host-side setting only: it applies to passes enqueued after the call.
 */
int cdsgd_plan_set_max_workgroups(cdsgd_plan *plan, int max_workgroups);

/*
 * Let correction and warm-up passes sum the workers' 32-bit gradients themselves
 * (Alg. 1, else-branch and WARMUP; the sum of eq. 1) instead of reading agg_full:
 * one launch then reads W and the N gradients and writes W and W_loc.
 *   peer_grads  host array [num_workers] of host arrays [num_tensors] of device
 *               pointers to fp32[n] (what the server would receive); row `self` is
 *               ignored (the own gradient is cdsgd_tensor.grad) and may be NULL.
 * Copies the pointers to the device (allocates on first use, synchronous copy);
 * the plan borrows the buffers.  May be called again to rebind: that rewrites the
 * pointer table the kernels read, so do not call it while a pass of this plan may
 * still be running.  With num_workers == 1 nothing is needed and the call is a no-op.
 */
int cdsgd_plan_bind_full_grads(cdsgd_plan *plan, const float *const *const *peer_grads);

/*
 * One pass of Alg. 1's WARMUP loop (i = 0 .. warmup_steps) for every tensor of the
 * plan: plain S-SGD on the global weights (eq. 1) with the fp32 sum of all
 * gradients (summed in the kernel if full gradients are bound, else agg_full;
 * CDSGD_ERR_NULL if the plan has neither).
 *   i <  warmup_steps - 1   w_local is not written
 *   i == warmup_steps - 1   w_local = the new global weights (the copy after the pull)
 *   i == warmup_steps       w_local = W - lr_local * grad, W being the global weights before
 *                           this pass (eq. 11).  For warmup_steps >= 1 that W is what the
 *                           previous pass copied into w_local; for warmup_steps == 0 Alg. 1
 *                           has no earlier pass to make the copy, and the base is still the
 *                           global weight: w_local is write-only in every pass, its content
 *                           before the call is never read.
 * i outside [0, warmup_steps] is CDSGD_ERR_PARAM.
 */
int cdsgd_step_warmup(cdsgd_plan *plan, long i, long warmup_steps, float lr_local, float lr_global,
                      void *hip_stream);

/*
 * Alg. 1 as a whole, as a counter around cdsgd_step_warmup and cdsgd_step_fused:
 * iterations 0 .. warmup_steps are WARMUP passes, iteration warmup_steps + 1 + c is
 * FormalTraining's pass with count = c.  Every formal pass, the first one included,
 * computes w_local from the global weights as they stand before the pass (eq. 11), not
 * from what the last warm-up pass left in w_local.  The trainer borrows the plan
 * (destroy the trainer first) and owns nothing on the device.
 */
typedef enum { CDSGD_PASS_WARMUP = 0, CDSGD_PASS_COMPRESSED = 1, CDSGD_PASS_CORRECTION = 2 } cdsgd_pass;
typedef struct cdsgd_trainer cdsgd_trainer;

int cdsgd_trainer_create(cdsgd_plan *plan, long warmup_steps, int k, float threshold, float lr_local,
                         float lr_global, cdsgd_trainer **out);
/* Enqueue the next iteration; *pass_kind (may be NULL) receives a cdsgd_pass.  On an
 * error nothing is enqueued and the iteration number does not advance. */
int cdsgd_trainer_step(cdsgd_trainer *trainer, void *hip_stream, int *pass_kind);
/* Number of iterations enqueued so far (-1 for NULL). */
long cdsgd_trainer_iteration(const cdsgd_trainer *trainer);
int cdsgd_trainer_destroy(cdsgd_trainer *trainer);

/*
 * Measurement aid, not part of the method: a bare streaming kernel that reads num_reads (0..17) fp32
 * buffers of n elements and writes num_writes (0..3) others (the sum of what it read, added in the
 * order given, plus the stream's index), with the loads, stores and launch shape of the passes on
 * 32-bit gradients and no other arithmetic.  Up to 3 read streams are loaded together; beyond that
 * they are read one after the other, the way a correction pass reads the workers' gradients.  A
 * benchmark uses it to state what the memory system gives a kernel with a given mix of read and
 * write streams, next to what the fused kernels reach with theirs.
 *   CDSGD_ERR_PARAM for counts outside those ranges or both zero, CDSGD_ERR_SIZE for n not a positive
 *   multiple of 256, CDSGD_ERR_ALIAS when a written buffer overlaps another buffer.
 *   reads / writes  HOST arrays of DEVICE pointers to fp32[n], 16-byte aligned, pairwise distinct
 *   n               a multiple of 256
 *   sink            device buffer of n / 256 floats, needed (and practically never written) when
 *                   num_writes == 0; may be NULL otherwise
 *   lds_bytes       LDS that every one-wave workgroup asks for and never touches (0 .. 65536, else
 *                   CDSGD_ERR_PARAM): it bounds the waves resident per compute unit at
 *                   163840 / lds_bytes, the knob the library's own single-wave kernels are launched
 *                   with; 0 = no bound (32 waves)
 */
int cdsgd_probe_streams(const float *const *reads, int num_reads, float *const *writes, int num_writes,
                        size_t n, float *sink, unsigned lds_bytes, void *hip_stream);

/*
 * cdsgd_step_fused for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same pass, same results
 * and same argument checks as cdsgd_plan_create_typed followed by cdsgd_step_fused on that
 * plan, but no plan: the layer list and the peers' pointers are passed on every call, and
 * the tables a plan would keep in memory of its own (tensor descriptors, chunk table,
 * peers' pointer table) are written, on `hip_stream` and by small kernels whose data travel
 * in their arguments, into one static device array of about 4.6 MiB that the library holds
 * on every GPU it runs on until the process ends.  The call makes no allocation, free or
 * host-to-device copy call; the first call on a device looks up the array's address (make
 * that call outside a graph capture).
 *   limits      num_tensors <= CDSGD_STATIC_MAX_TENSORS and
 *               sum over tensors of ceil(n / CDSGD_STATIC_CHUNK_ELEMS) <= CDSGD_STATIC_MAX_CHUNKS
 *               (up to 2^31 elements in all): CDSGD_ERR_SIZE beyond that.
 *   correction  passes (step % k == 0) read agg_full of every tensor (CDSGD_ERR_NULL if one is
 *               missing and num_workers > 1); bound full gradients and per-tensor thresholds are
 *               features of a plan and are not available here.
 *   sharing     every call on a GPU uses that GPU's one array: calls on the same stream are
 *               ordered and safe; calls that may overlap on one GPU (different streams, or
 *               different host threads on different streams) race on the tables and must be
 *               ordered by the caller.  Plans are not affected.
 * The tables are rebuilt on every call (a few small launches before the pass itself), so a
 * plan remains the faster form for a layer list that is stepped many times.
 */
#define CDSGD_STATIC_MAX_TENSORS 1024
#define CDSGD_STATIC_MAX_CHUNKS 524288
#define CDSGD_STATIC_CHUNK_ELEMS 4096
int cdsgd_step_fused_static(const cdsgd_tensor *tensors, int num_tensors,
                            const uint32_t *const *const *peers, int num_workers, int self,
                            int grad_dtype, long step, int k, float threshold, float lr_local,
                            float lr_global, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* CDSGD_H */
