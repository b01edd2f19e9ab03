// CD-SGD per-step data-parallel hot path for gfx950 (MI355X): the C ABI and the host side of every
// entry point.  One translation unit; the kernels are in the .hpp files beside this one:
//   tuning.hpp          build-time knobs (launch shapes, cache policy)
//   device_common.hpp   chunk geometry, 128-bit loads / stores, 16-bit widening, the quantiser
//   device_tables.hpp   extents, tensor descriptors, chunk table
//   kernels_tensor.hpp  single-tensor kernels (quantise-and-pack, decode-and-sum, update)
//   kernels_sparse.hpp  sparse form of a packed stream
//   kernels_probe.hpp   bare streaming kernel (measurement aid)
//   kernels_fused.hpp   passes over a layer list: fused compressed pass, passes on 32-bit gradients
//   kernels_static.hpp  tables built on the device for the entry point that allocates nothing
//
// Work decomposition.  The unit of work of one lane is a "quad": four
// consecutive fp32 elements = one 128-bit load/store per buffer = one byte of
// the packed stream (four 2-bit codes; element e of a tensor is bits
// [2(e%4)+1 : 2(e%4)] of packed byte e/4, which is the little-endian view of
// the 32-bit-word layout in cdsgd.h).  A tensor is cut into "chunks" of 1024
// quads (4096 elements, 1 KiB of a packed stream); the chunk table of a plan
// lists (tensor, chunk) pairs, and only a tensor's last chunk can be ragged.
//   * The kernels over a layer list work on "pieces" of a chunk, one quad per
//     lane: 256-lane workgroups for the compressed pass (the peers' codes
//     come in through LDS, 128 bits per lane and 16 peers per instruction),
//     single waves for the passes on 32-bit gradients.
//   * Of the single-tensor kernels, decode-and-sum gives a chunk to a
//     workgroup of kBlock lanes, lane `tid` taking quads j*kBlock + tid;
//     quantise-and-pack and the update work in single-wave pieces.
// Either way every wave instruction on an fp32 buffer touches one contiguous
// 1 KiB span: all traffic is fully coalesced.
//
// The path is elementwise and HBM-bound: no MFMA.  Each of grad / residual /
// w_global is read once and each of residual / w_global / w_local is written
// once per step.

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "cdsgd.h"

#include "tuning.hpp"
#include "device_common.hpp"
#include "device_tables.hpp"
#include "kernels_tensor.hpp"
#include "kernels_sparse.hpp"
#include "kernels_probe.hpp"
#include "kernels_fused.hpp"
#include "kernels_static.hpp"

// The tables of cdsgd_step_fused_static live here (about 4.6 MiB on every GPU the library
// runs on, until the process ends).  In host code this name is only a handle for
// hipGetSymbolAddress; the device address is looked up once per device (static_scratch).
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

namespace {

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
// LDS that the single-wave kernels ask for at launch and never touch: it bounds the waves resident per
// compute unit (160 KiB / bytes).  With all 32 resident, more requests queue in front of HBM than it takes
// to keep it busy, and a mix of reads and writes is then served more slowly.  Measured (2^27 elements or the
// VGG-16-shaped list; TB/s at 32 / 26 / 22 / 20 / 17 / 16 / 13 / 10 resident waves):
//   correction pass with agg_full   6.42-6.45 / 6.40 / 6.51 / 6.66-6.67 / 6.55 / 6.55-6.60 / 6.41 / 5.88
//   quantise-and-pack               6.71 / 6.72 / - / 6.83 / - / 6.88 / 6.09 / 5.10
//   update, both rules              6.36 / 6.34 / - / 6.55 / - / 6.50 / 6.55 / 6.18
//   correction pass, sum in kernel  6.19 / 6.39-6.41 / 6.35 / 6.24 / - / 5.97
// eq. 11 alone and the compressed pass (whose workgroups already hold 4-16 KiB of staged codes) lose with
// any bound and get none.  The same bound stated to the compiler instead (amdgpu_waves_per_eu with a maximum of
// 5) gives 6.55 and 6.45 TB/s on the first and the third line: most of the gain, not all of it.  While a
// pass launched this way runs it holds the compute units' LDS, so a kernel of another stream that needs
// LDS waits for it; a pass with a workgroup limit (cdsgd_plan_set_max_workgroups), which is meant to run
// beside other kernels, is launched without the bound.
constexpr unsigned kLdsFor20Waves = 8192;
constexpr unsigned kLdsFor26Waves = 6144;

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Do [a, a + na) and [b, b + nb) share a byte?  (NULL never overlaps.)
inline bool overlap2(const void *a, size_t na, const void *b, size_t nb)
{
    if (!a || !b) return false;
    const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
    return x < y ? y - x < na : x - y < nb;
}

// Do the byte ranges [a, a + bytes) and [b, b + bytes) share a byte?  (NULL never overlaps.)
inline bool overlap(const void *a, const void *b, size_t bytes)
{
    if (!a || !b) return false;
    const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
    return x < y ? y - x < bytes : x - y < bytes;
}

inline unsigned long long packed_bytes_of(size_t n) { return 4ull * ((n + 15) / 16); }

// Chunks needed to cover a tensor's packed stream (which covers its elements):
// n / kChunkElems full ones, plus one for the ragged end if there is one.
inline unsigned long long chunks_of(size_t n) { return (packed_bytes_of(n) + kChunkQuads - 1) / kChunkQuads; }

inline Extent extent_of(size_t n)
{
    Extent e;
    const unsigned long long full = n / kChunkElems;
    e.full_chunks = (unsigned)full;
    e.tail_elems = (unsigned)(n - full * kChunkElems);
    e.tail_bytes = (unsigned)(packed_bytes_of(n) - full * kChunkQuads);
    e.pad_ = 0;
    return e;
}

// The same in units of `unit_quads` quads (the single-tensor kernels' pieces).
inline unsigned long long units_of(size_t n, unsigned unit_quads)
{
    return (packed_bytes_of(n) + unit_quads - 1) / unit_quads;
}

inline Extent extent_of_units(size_t n, unsigned unit_quads)
{
    Extent e;
    const unsigned long long full = n / (4ull * unit_quads);
    e.full_chunks = (unsigned)full;
    e.tail_elems = (unsigned)(n - full * 4ull * unit_quads);
    e.tail_bytes = (unsigned)(packed_bytes_of(n) - full * unit_quads);
    e.pad_ = 0;
    return e;
}

// Most chunks (or segments) a tensor or a layer list may have: a launch of one workgroup of up to
// 1024 lanes per chunk stays below 2^32 threads (1.7e10 elements).
constexpr unsigned long long kMaxGrid = 0xFFFFFFFFull / 1024;
constexpr unsigned kQuantLanes = 64;   // lanes = quads of a piece of k_quantize_pack
constexpr unsigned kUpdateLanes = 64;  // ... and of k_update
// lanes of k_decode_sum's workgroup (one chunk): measured on 2^27 elements, N = 16, count form 6.03 TB/s with
// 512 lanes and 5.78 with 256; literal chain 4.66 with 512 and 5.40 with 256 (more workgroups resident to
// hide its arithmetic)
constexpr unsigned kDecodeLanesCount = 512, kDecodeLanesChain = 256;
// ... and of k_decode_sum_sparse's: 256 either way (count form, nothing sent / every word sent: 4.15 / 5.66 TB/s of
// the bytes moved against 3.76 / 4.53 with 512)
constexpr unsigned kSparseLanes = 256;

// A threshold 2^e (moderate e): every multiple m*t, |m| <= 2*CDSGD_MAX_WORKERS, is exact.
inline bool is_pow2_threshold(float t)
{
    int e = 0;
    const float m = std::frexp(t, &e);
    return m == 0.5f && e > -100 && e < 100;
}

inline bool good_threshold(float t) { return std::isfinite(t) && t > 0.0f; }

inline bool good_step_params(long step, int k, float threshold, float lr_local, float lr_global)
{
    return k >= 1 && step >= 0 && good_threshold(threshold) && std::isfinite(lr_local) && std::isfinite(lr_global);
}

inline int launch_status()
{
    return hipGetLastError() == hipSuccess ? CDSGD_OK : CDSGD_ERR_DEVICE;
}

}  // namespace

// What a pass needs to know about a layer list: device tables and a few host-side facts.
// A plan owns one (tables in memory it allocated); the entry point that allocates nothing
// builds one on the stack, its tables in the library's static device array.
struct PlanTables {
    TensorDesc *tensors = nullptr;
    ChunkRef *chunks = nullptr;
    const uint8_t **peers = nullptr;    // [num_tensors][num_workers - 1]
    const void **peer_grads = nullptr;  // same shape, or null: correction passes read agg_full
    int num_tensors = 0;
    int num_workers = 0;
    int self = 0;
    unsigned first_chunk = 0;           // a pass covers chunks [first_chunk, first_chunk + num_chunks) of the table
    unsigned num_chunks = 0;
    bool has_agg_full = false;
    int grad_type = kGradF32;          // element type of grad and of the bound peer gradients
    bool own_thresholds = false;       // every tensor carries its own threshold
    bool own_thresholds_pow2 = false;  // ... and all of them are powers of two
    unsigned max_workgroups = 0;       // > 0: launch at most this many workgroups (they take several chunks each)
    bool peers_sparse = false;         // the peers' streams are in the sparse form (cdsgd_plan_set_peer_format)

    // Workgroups of `lanes` lanes to launch for `units` units of work (pieces of chunks): one per unit,
    // unless the plan has a limit or the launch would pass 2^32 - 1 threads (the kernels walk the units
    // with the grid's stride, so fewer workgroups than units is always correct).
    const ChunkRef *chunk_table() const { return chunks + first_chunk; }

    unsigned grid_size(unsigned long long units, unsigned lanes) const
    {
        unsigned long long cap = 0xFFFFFFFFull / lanes;
        if (max_workgroups != 0 && max_workgroups < cap) cap = max_workgroups;
        return (unsigned)(units < cap ? units : cap);
    }
};

struct cdsgd_plan : PlanTables {
    void *device_block = nullptr;          // one allocation: tensors, chunks, peer pointers
    void *peer_grads_block = nullptr;      // second allocation, made by cdsgd_plan_bind_full_grads
    std::vector<TensorDesc> host_tensors;  // host copy of the descriptor table (for cdsgd_plan_set_thresholds)
    std::vector<unsigned> chunk_start;     // chunk_start[i] = first chunk of tensor i; num_tensors + 1 entries
};

struct cdsgd_trainer {
    cdsgd_plan *plan = nullptr;
    long warmup_steps = 0;
    int k = 1;
    float threshold = 0.0f, lr_local = 0.0f, lr_global = 0.0f;
    long iteration = 0;
};

namespace {

// Host-side checks of a layer list and its peers (no HIP call): what cdsgd_plan_create_typed
// and cdsgd_step_fused_static share.  Returns the number of chunks and whether every tensor
// has an agg_full buffer.
int check_layer_list(const cdsgd_tensor *tensors, int num_tensors, const uint32_t *const *const *peers,
                     int num_workers, int self, int grad_dtype, unsigned long long *total_chunks_out,
                     bool *all_agg_out)
{
    if (!tensors) return CDSGD_ERR_NULL;
    if (grad_dtype != CDSGD_GRAD_F32 && grad_dtype != CDSGD_GRAD_BF16 && grad_dtype != CDSGD_GRAD_F16)
        return CDSGD_ERR_PARAM;
    const size_t grad_elem = grad_dtype == CDSGD_GRAD_F32 ? 4 : 2;
    if (num_tensors < 1) return CDSGD_ERR_SIZE;
    if (num_workers < 1 || num_workers > CDSGD_MAX_WORKERS || self < 0 || self >= num_workers)
        return CDSGD_ERR_WORKERS;
    if (num_workers > 1 && !peers) return CDSGD_ERR_NULL;
    unsigned long long total_chunks = 0;
    bool all_agg = true;
    for (int i = 0; i < num_tensors; ++i) {
        const cdsgd_tensor &t = tensors[i];
        if (!t.w_global || !t.w_local || !t.residual || !t.grad || !t.packed_self) return CDSGD_ERR_NULL;
        if (t.n == 0 || chunks_of(t.n) > kMaxGrid) return CDSGD_ERR_SIZE;
        if (!aligned(t.w_global, 16) || !aligned(t.w_local, 16) || !aligned(t.residual, 16) ||
            !aligned(t.grad, 16) || !aligned(t.agg_full, 16) || !aligned(t.packed_self, 4))
            return CDSGD_ERR_ALIGN;
        const size_t fb = t.n * sizeof(float), gb = t.n * grad_elem, pb = (size_t)packed_bytes_of(t.n);
        if (overlap(t.w_global, t.w_local, fb) || overlap(t.w_global, t.residual, fb) ||
            overlap(t.w_local, t.residual, fb) || overlap(t.agg_full, t.w_global, fb) ||
            overlap(t.agg_full, t.w_local, fb) || overlap2(t.grad, gb, t.residual, fb) ||
            overlap2(t.grad, gb, t.w_global, fb) || overlap2(t.grad, gb, t.w_local, fb) ||
            overlap2(t.packed_self, pb, t.w_global, fb) || overlap2(t.packed_self, pb, t.w_local, fb) ||
            overlap2(t.packed_self, pb, t.residual, fb) || overlap2(t.packed_self, pb, t.grad, gb) ||
            overlap2(t.packed_self, pb, t.agg_full, fb))
            return CDSGD_ERR_ALIAS;
        all_agg = all_agg && t.agg_full != nullptr;
        total_chunks += chunks_of(t.n);
        if (total_chunks > kMaxGrid) return CDSGD_ERR_SIZE;
    }
    for (int j = 0; j < num_workers; ++j) {
        if (j == self) continue;
        if (!peers[j]) return CDSGD_ERR_NULL;
        for (int i = 0; i < num_tensors; ++i) {
            if (!peers[j][i]) return CDSGD_ERR_NULL;
            if (!aligned(peers[j][i], 4)) return CDSGD_ERR_ALIGN;
            // a peer's stream is read while this tensor's outputs are written
            const cdsgd_tensor &t = tensors[i];
            const size_t fb = t.n * sizeof(float), pb = (size_t)packed_bytes_of(t.n);
            if (overlap2(peers[j][i], pb, t.w_global, fb) || overlap2(peers[j][i], pb, t.w_local, fb) ||
                overlap2(peers[j][i], pb, t.residual, fb) || overlap2(peers[j][i], pb, t.packed_self, pb))
                return CDSGD_ERR_ALIAS;
        }
    }
    *total_chunks_out = total_chunks;
    *all_agg_out = all_agg;
    return CDSGD_OK;
}

TensorDesc make_desc(const cdsgd_tensor &t)
{
    TensorDesc d;
    d.w_global = t.w_global;
    d.w_local = t.w_local;
    d.residual = t.residual;
    d.grad = t.grad;
    d.packed_self = reinterpret_cast<uint8_t *>(t.packed_self);
    d.agg_full = t.agg_full;
    d.ext = extent_of(t.n);
    d.threshold = 0.0f;
    d.pad_ = 0;
    return d;
}

// Launch one full-gradient pass (see k_fused_full) for a plan.
int launch_full_pass(const PlanTables *plan, int local_mode, float lr_local, float lr_global, void *hip_stream)
{
    const bool sum = plan->peer_grads != nullptr || plan->num_workers == 1;
    if (!sum && !plan->has_agg_full) return CDSGD_ERR_NULL;
    const float scale = lr_global / (float)plan->num_workers;
    hipStream_t s = (hipStream_t)hip_stream;
    const unsigned long long num_pieces = (unsigned long long)plan->num_chunks * kPiecesPerChunk;
    const dim3 grid(plan->grid_size(num_pieces, kFullBlock)), block(kFullBlock);
    const int np = plan->num_workers - 1;
    // a pass with a workgroup limit is meant to share the GPU with other kernels: it leaves the LDS to them
    const unsigned lds_plain = plan->max_workgroups ? 0u : kLdsFor20Waves;
    const unsigned lds_sum = plan->max_workgroups ? 0u : kLdsFor26Waves;
#define CDSGD_LAUNCH_FULL_T(SUM, LOCAL, GT)                                                                    \
    hipLaunchKernelGGL((k_fused_full<SUM, LOCAL, GT>), grid, block, (SUM ? lds_sum : lds_plain), s,              \
                       plan->tensors, plan->chunk_table(),                                                      \
                       num_pieces, plan->peer_grads, np, plan->self, lr_local, scale)
#define CDSGD_LAUNCH_FULL(SUM, LOCAL)                                                                          \
    do {                                                                                                       \
        if (plan->grad_type == kGradBF16) CDSGD_LAUNCH_FULL_T(SUM, LOCAL, kGradBF16);                          \
        else if (plan->grad_type == kGradF16) CDSGD_LAUNCH_FULL_T(SUM, LOCAL, kGradF16);                       \
        else CDSGD_LAUNCH_FULL_T(SUM, LOCAL, kGradF32);                                                        \
    } while (0)
    if (sum) {
        if (local_mode == kLocalNone) CDSGD_LAUNCH_FULL(true, kLocalNone);
        else if (local_mode == kLocalCopy) CDSGD_LAUNCH_FULL(true, kLocalCopy);
        else CDSGD_LAUNCH_FULL(true, kLocalRule);
    } else {
        if (local_mode == kLocalNone) CDSGD_LAUNCH_FULL(false, kLocalNone);
        else if (local_mode == kLocalCopy) CDSGD_LAUNCH_FULL(false, kLocalCopy);
        else CDSGD_LAUNCH_FULL(false, kLocalRule);
    }
#undef CDSGD_LAUNCH_FULL
#undef CDSGD_LAUNCH_FULL_T
    return launch_status();
}

}  // namespace

#ifndef CDSGD_BUILD_ID_HEX
#define CDSGD_BUILD_ID_HEX "0000000000000000"
#endif

extern "C" {

size_t cdsgd_packed_words(size_t n) { return (n + 15) / 16; }

// The marker in front makes the identity findable in the file without loading it.
const char *cdsgd_build_id(void)
{
    static const char id[] = "CDSGD_BUILD_ID=" CDSGD_BUILD_ID_HEX;
    return id + 15;
}

const char *cdsgd_status_string(int status)
{
    switch (status) {
    case CDSGD_OK: return "ok";
    case CDSGD_ERR_NULL: return "a required pointer is NULL";
    case CDSGD_ERR_SIZE:
        return "bad size (zero elements, no tensors, too large for one launch, or beyond the limits of "
               "cdsgd_step_fused_static's tables)";
    case CDSGD_ERR_PARAM: return "bad parameter (threshold, k, step or learning rate)";
    case CDSGD_ERR_ALIGN: return "pointer not aligned (fp32 buffers 16 bytes, packed buffers 4 bytes)";
    case CDSGD_ERR_WORKERS: return "bad worker count or worker index";
    case CDSGD_ERR_DEVICE: return "a HIP call failed";
    case CDSGD_ERR_ALIAS: return "buffers that must be distinct overlap";
    default: return "unknown status";
    }
}

int cdsgd_quantize_pack(const float *grad, float *residual, uint32_t *packed, size_t n, float threshold,
                        void *hip_stream)
{
    if (!grad || !residual || !packed) return CDSGD_ERR_NULL;
    if (n == 0 || units_of(n, kQuantLanes) > 0xFFFFFFFFull / kQuantLanes) return CDSGD_ERR_SIZE;
    if (!good_threshold(threshold)) return CDSGD_ERR_PARAM;
    if (!aligned(grad, 16) || !aligned(residual, 16) || !aligned(packed, 4)) return CDSGD_ERR_ALIGN;
    if (overlap(grad, residual, n * sizeof(float)) ||
        overlap2(packed, (size_t)packed_bytes_of(n), grad, n * sizeof(float)) ||
        overlap2(packed, (size_t)packed_bytes_of(n), residual, n * sizeof(float)))
        return CDSGD_ERR_ALIAS;
    hipLaunchKernelGGL(k_quantize_pack<kQuantLanes>, dim3((unsigned)units_of(n, kQuantLanes)), dim3(kQuantLanes), kLdsFor20Waves,
                       (hipStream_t)hip_stream, grad, residual, reinterpret_cast<uint8_t *>(packed),
                       extent_of_units(n, kQuantLanes), threshold);
    return launch_status();
}

int cdsgd_decode_sum(const uint32_t *const *packed, int num_workers, float *agg, size_t n, float threshold,
                     void *hip_stream)
{
    if (!packed || !agg) return CDSGD_ERR_NULL;
    if (n == 0 || chunks_of(n) > kMaxGrid) return CDSGD_ERR_SIZE;
    if (!good_threshold(threshold)) return CDSGD_ERR_PARAM;
    if (num_workers < 1 || num_workers > CDSGD_MAX_WORKERS) return CDSGD_ERR_WORKERS;
    for (int j = 0; j < num_workers; ++j)
        if (!packed[j]) return CDSGD_ERR_NULL;
    if (!aligned(agg, 16)) return CDSGD_ERR_ALIGN;
    for (int j = 0; j < num_workers; ++j)
        if (!aligned(packed[j], 4)) return CDSGD_ERR_ALIGN;
    for (int j = 0; j < num_workers; ++j)
        if (overlap2(packed[j], (size_t)packed_bytes_of(n), agg, n * sizeof(float))) return CDSGD_ERR_ALIAS;
    StreamTable tab;
    std::memset(&tab, 0, sizeof(tab));
    for (int j = 0; j < num_workers; ++j) tab.p[j] = reinterpret_cast<const uint8_t *>(packed[j]);
    const float bias_t = -(2.0f * (float)num_workers) * threshold;
    const unsigned grid = (unsigned)chunks_of(n);
    if (is_pow2_threshold(threshold))
        hipLaunchKernelGGL((k_decode_sum<true, kDecodeLanesCount>), dim3(grid), dim3(kDecodeLanesCount), 0, (hipStream_t)hip_stream, tab,
                           num_workers, agg, extent_of(n), threshold, bias_t);
    else
        hipLaunchKernelGGL((k_decode_sum<false, kDecodeLanesChain>), dim3(grid), dim3(kDecodeLanesChain), 0, (hipStream_t)hip_stream, tab,
                           num_workers, agg, extent_of(n), threshold, bias_t);
    return launch_status();
}

int cdsgd_update(float *w_global, float *w_local, const float *grad_local, const float *agg, size_t n,
                 float lr_local, float lr_global, int num_workers, void *hip_stream)
{
    const bool local = w_local != nullptr || grad_local != nullptr;
    const bool global = agg != nullptr;
    if (!w_global) return CDSGD_ERR_NULL;
    if (local && (!w_local || !grad_local)) return CDSGD_ERR_NULL;
    if (!local && !global) return CDSGD_ERR_NULL;
    if (n == 0 || units_of(n, kUpdateLanes) > 0xFFFFFFFFull / kUpdateLanes) return CDSGD_ERR_SIZE;
    if (!std::isfinite(lr_local) || !std::isfinite(lr_global)) return CDSGD_ERR_PARAM;
    if (num_workers < 1 || num_workers > CDSGD_MAX_WORKERS) return CDSGD_ERR_WORKERS;
    if (!aligned(w_global, 16) || !aligned(w_local, 16) || !aligned(grad_local, 16) || !aligned(agg, 16))
        return CDSGD_ERR_ALIGN;
    if (overlap(w_global, w_local, n * sizeof(float)) || overlap(w_local, grad_local, n * sizeof(float)) ||
        overlap(w_local, agg, n * sizeof(float)) || overlap(w_global, grad_local, n * sizeof(float)) ||
        overlap(w_global, agg, n * sizeof(float)))
        return CDSGD_ERR_ALIAS;
    const float scale = lr_global / (float)num_workers;
    hipStream_t s = (hipStream_t)hip_stream;
    const dim3 grid((unsigned)units_of(n, kUpdateLanes)), block(kUpdateLanes);
    const Extent pieces = extent_of_units(n, kUpdateLanes);
    if (local && global)
        hipLaunchKernelGGL((k_update<true, true>), grid, block, kLdsFor20Waves, s, w_global, w_local, grad_local, agg, pieces, lr_local, scale);
    else if (local)
        hipLaunchKernelGGL((k_update<true, false>), grid, block, 0, s, w_global, w_local, grad_local, agg, pieces, lr_local, scale);
    else
        hipLaunchKernelGGL((k_update<false, true>), grid, block, 0, s, w_global, w_local, grad_local, agg, pieces, lr_local, scale);
    return launch_status();
}

int cdsgd_plan_create(const cdsgd_tensor *tensors, int num_tensors, const uint32_t *const *const *peers,
                      int num_workers, int self, cdsgd_plan **out)
{
    return cdsgd_plan_create_typed(tensors, num_tensors, peers, num_workers, self, CDSGD_GRAD_F32, out);
}

int cdsgd_plan_create_typed(const cdsgd_tensor *tensors, int num_tensors, const uint32_t *const *const *peers,
                            int num_workers, int self, int grad_dtype, cdsgd_plan **out)
{
    if (!out) return CDSGD_ERR_NULL;
    *out = nullptr;
    unsigned long long total_chunks = 0;
    bool all_agg = true;
    const int rc = check_layer_list(tensors, num_tensors, peers, num_workers, self, grad_dtype, &total_chunks, &all_agg);
    if (rc != CDSGD_OK) return rc;
    const int num_peers = num_workers - 1;

    // host image of the device block
    const size_t bytes_t = sizeof(TensorDesc) * (size_t)num_tensors;
    const size_t bytes_c = sizeof(ChunkRef) * (size_t)total_chunks;
    const size_t bytes_p = sizeof(const uint8_t *) * (size_t)num_tensors * (size_t)(num_peers > 0 ? num_peers : 1);
    const size_t off_c = (bytes_t + 255) & ~(size_t)255;
    const size_t off_p = (off_c + bytes_c + 255) & ~(size_t)255;
    const size_t total = off_p + bytes_p;
    std::vector<unsigned char> image(total, 0);
    TensorDesc *ht = reinterpret_cast<TensorDesc *>(image.data());
    ChunkRef *hc = reinterpret_cast<ChunkRef *>(image.data() + off_c);
    const uint8_t **hp = reinterpret_cast<const uint8_t **>(image.data() + off_p);
    size_t ci = 0;
    std::vector<unsigned> chunk_start((size_t)num_tensors + 1, 0u);
    for (int i = 0; i < num_tensors; ++i) {
        const cdsgd_tensor &t = tensors[i];
        ht[i] = make_desc(t);
        const unsigned nc = (unsigned)chunks_of(t.n);
        chunk_start[(size_t)i + 1] = chunk_start[(size_t)i] + nc;
        for (unsigned c = 0; c < nc; ++c) {
            hc[ci].tensor = (unsigned)i;
            hc[ci].chunk = c;
            ++ci;
        }
        int slot = 0;
        for (int j = 0; j < num_workers; ++j) {
            if (j == self) continue;
            hp[(size_t)i * (size_t)num_peers + (size_t)slot] = reinterpret_cast<const uint8_t *>(peers[j][i]);
            ++slot;
        }
    }

    cdsgd_plan *plan = new (std::nothrow) cdsgd_plan;
    if (!plan) return CDSGD_ERR_DEVICE;
    if (hipMalloc(&plan->device_block, total) != hipSuccess) {
        (void)hipGetLastError();
        delete plan;
        return CDSGD_ERR_DEVICE;
    }
    if (hipMemcpy(plan->device_block, image.data(), total, hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipFree(plan->device_block);
        delete plan;
        return CDSGD_ERR_DEVICE;
    }
    unsigned char *base = static_cast<unsigned char *>(plan->device_block);
    plan->tensors = reinterpret_cast<TensorDesc *>(base);
    plan->chunks = reinterpret_cast<ChunkRef *>(base + off_c);
    plan->peers = reinterpret_cast<const uint8_t **>(base + off_p);
    plan->num_tensors = num_tensors;
    plan->num_workers = num_workers;
    plan->self = self;
    plan->num_chunks = (unsigned)total_chunks;
    plan->has_agg_full = all_agg;
    plan->grad_type = grad_dtype;
    plan->host_tensors.assign(ht, ht + num_tensors);
    plan->chunk_start.swap(chunk_start);
    *out = plan;
    return CDSGD_OK;
}

int cdsgd_plan_destroy(cdsgd_plan *plan)
{
    if (!plan) return CDSGD_OK;
    int rc = CDSGD_OK;
    if (plan->device_block && hipFree(plan->device_block) != hipSuccess) {
        (void)hipGetLastError();
        rc = CDSGD_ERR_DEVICE;
    }
    if (plan->peer_grads_block && hipFree(plan->peer_grads_block) != hipSuccess) {
        (void)hipGetLastError();
        rc = CDSGD_ERR_DEVICE;
    }
    delete plan;
    return rc;
}

namespace {

// One pass of FormalTraining's loop; with_local = false leaves eq. 11 out (split form).
int launch_formal_pass(const PlanTables *plan, long step, int k, float threshold, float lr_local, float lr_global,
                       bool with_local, void *hip_stream)
{
    if (!plan) return CDSGD_ERR_NULL;
    if (!good_step_params(step, k, threshold, lr_local, lr_global)) return CDSGD_ERR_PARAM;
    const bool compressed = (step % k) != 0;
    if (!compressed)
        return launch_full_pass(plan, with_local ? kLocalRule : kLocalNone, lr_local, lr_global, hip_stream);
    const float scale = lr_global / (float)plan->num_workers;
    hipStream_t s = (hipStream_t)hip_stream;
    const int num_peers = plan->num_workers - 1;
    const unsigned waves = num_peers <= kFewPeers ? 1u : kPieceWavesMany;
    const bool many = num_peers > 16;  // count form: the kernel compiled for more waves per SIMD
    const unsigned long long num_pieces = (unsigned long long)plan->num_chunks * (kChunkQuads / (64u * waves));
    const dim3 grid(plan->grid_size(num_pieces, 64u * waves)), block(64u * waves);
#define CDSGD_LAUNCH_COMPRESSED_S(W, POW2, LOCAL, GT, SPARSE)                                                  \
    hipLaunchKernelGGL((k_fused_compressed<W, POW2, LOCAL, GT, SPARSE>), grid, block, 0, s, plan->tensors,      \
                       plan->chunk_table(), num_pieces, plan->peers, num_peers, plan->self, threshold, lr_local, \
                       scale)
#define CDSGD_LAUNCH_COMPRESSED_M(LOCAL, GT, SPARSE)                                                           \
    hipLaunchKernelGGL((k_fused_compressed_many<LOCAL, GT, SPARSE>), grid, block, 0, s, plan->tensors,          \
                       plan->chunk_table(), num_pieces, plan->peers, num_peers, plan->self, threshold, lr_local, \
                       scale)
#define CDSGD_LAUNCH_COMPRESSED_W(W, POW2, LOCAL, GT)                                                          \
    do {                                                                                                       \
        if (POW2 && many) {                                                                                    \
            if (plan->peers_sparse) CDSGD_LAUNCH_COMPRESSED_M(LOCAL, GT, true);                                 \
            else CDSGD_LAUNCH_COMPRESSED_M(LOCAL, GT, false);                                                   \
        } else if (plan->peers_sparse) CDSGD_LAUNCH_COMPRESSED_S(W, POW2, LOCAL, GT, true);                     \
        else CDSGD_LAUNCH_COMPRESSED_S(W, POW2, LOCAL, GT, false);                                              \
    } while (0)
#define CDSGD_LAUNCH_COMPRESSED_T(POW2, LOCAL, GT)                                                            \
    do {                                                                                                       \
        if (waves == 1u) CDSGD_LAUNCH_COMPRESSED_W(1u, POW2, LOCAL, GT);                                        \
        else CDSGD_LAUNCH_COMPRESSED_W(kPieceWavesMany, POW2, LOCAL, GT);                                       \
    } while (0)
#define CDSGD_LAUNCH_COMPRESSED(POW2, LOCAL)                                                                  \
    do {                                                                                                       \
        if (plan->grad_type == kGradBF16) CDSGD_LAUNCH_COMPRESSED_T(POW2, LOCAL, kGradBF16);                   \
        else if (plan->grad_type == kGradF16) CDSGD_LAUNCH_COMPRESSED_T(POW2, LOCAL, kGradF16);                \
        else CDSGD_LAUNCH_COMPRESSED_T(POW2, LOCAL, kGradF32);                                                 \
    } while (0)
    // the count form of the decode needs every threshold in use to be a power of two
    const bool pow2 = plan->own_thresholds ? plan->own_thresholds_pow2 : is_pow2_threshold(threshold);
    if (pow2) {
        if (with_local) CDSGD_LAUNCH_COMPRESSED(true, true);
        else CDSGD_LAUNCH_COMPRESSED(true, false);
    } else {
        if (with_local) CDSGD_LAUNCH_COMPRESSED(false, true);
        else CDSGD_LAUNCH_COMPRESSED(false, false);
    }
#undef CDSGD_LAUNCH_COMPRESSED
#undef CDSGD_LAUNCH_COMPRESSED_T
#undef CDSGD_LAUNCH_COMPRESSED_W
#undef CDSGD_LAUNCH_COMPRESSED_M
#undef CDSGD_LAUNCH_COMPRESSED_S
    return launch_status();
}

}  // namespace

int cdsgd_step_fused(cdsgd_plan *plan, long step, int k, float threshold, float lr_local, float lr_global,
                     void *hip_stream)
{
    return launch_formal_pass(plan, step, k, threshold, lr_local, lr_global, true, hip_stream);
}

namespace {

// eq. 11 alone over the chunks a PlanTables covers.
int launch_local_pass(const PlanTables *plan, float lr_local, void *hip_stream)
{
    if (!plan) return CDSGD_ERR_NULL;
    if (!std::isfinite(lr_local)) return CDSGD_ERR_PARAM;
    const unsigned long long num_pieces = (unsigned long long)plan->num_chunks * kPiecesPerChunk;
    const dim3 grid(plan->grid_size(num_pieces, kFullBlock)), block(kFullBlock);
    hipStream_t s = (hipStream_t)hip_stream;
#define CDSGD_LAUNCH_LOCAL(GT)                                                                                 \
    hipLaunchKernelGGL((k_fused_full<false, kLocalOnly, GT>), grid, block, 0, s, plan->tensors,                  \
                       plan->chunk_table(), num_pieces, (const void *const *)nullptr, 0, plan->self, lr_local,   \
                       0.0f)
    if (plan->grad_type == kGradBF16) CDSGD_LAUNCH_LOCAL(kGradBF16);
    else if (plan->grad_type == kGradF16) CDSGD_LAUNCH_LOCAL(kGradF16);
    else CDSGD_LAUNCH_LOCAL(kGradF32);
#undef CDSGD_LAUNCH_LOCAL
    return launch_status();
}

// The part of a plan's tables that covers tensors [first_tensor, first_tensor + num_tensors).
int slice_of_plan(const cdsgd_plan *plan, int first_tensor, int num_tensors, PlanTables *out)
{
    if (!plan) return CDSGD_ERR_NULL;
    if (first_tensor < 0 || num_tensors < 1 || first_tensor > plan->num_tensors - num_tensors) return CDSGD_ERR_PARAM;
    *out = *plan;  // the tables themselves are shared; only the range of chunks differs
    out->first_chunk = plan->chunk_start[(size_t)first_tensor];
    out->num_chunks = plan->chunk_start[(size_t)first_tensor + (size_t)num_tensors] - out->first_chunk;
    return CDSGD_OK;
}

}  // namespace

int cdsgd_step_local(cdsgd_plan *plan, float lr_local, void *hip_stream)
{
    return launch_local_pass(plan, lr_local, hip_stream);
}

int cdsgd_step_global(cdsgd_plan *plan, long step, int k, float threshold, float lr_global, void *hip_stream)
{
    return launch_formal_pass(plan, step, k, threshold, 0.0f, lr_global, false, hip_stream);
}

int cdsgd_step_fused_range(cdsgd_plan *plan, int first_tensor, int num_tensors, long step, int k, float threshold,
                           float lr_local, float lr_global, void *hip_stream)
{
    PlanTables part;
    const int rc = slice_of_plan(plan, first_tensor, num_tensors, &part);
    if (rc != CDSGD_OK) return rc;
    return launch_formal_pass(&part, step, k, threshold, lr_local, lr_global, true, hip_stream);
}

int cdsgd_step_local_range(cdsgd_plan *plan, int first_tensor, int num_tensors, float lr_local, void *hip_stream)
{
    PlanTables part;
    const int rc = slice_of_plan(plan, first_tensor, num_tensors, &part);
    if (rc != CDSGD_OK) return rc;
    return launch_local_pass(&part, lr_local, hip_stream);
}

int cdsgd_step_global_range(cdsgd_plan *plan, int first_tensor, int num_tensors, long step, int k, float threshold,
                            float lr_global, void *hip_stream)
{
    PlanTables part;
    const int rc = slice_of_plan(plan, first_tensor, num_tensors, &part);
    if (rc != CDSGD_OK) return rc;
    return launch_formal_pass(&part, step, k, threshold, 0.0f, lr_global, false, hip_stream);
}

int cdsgd_plan_bind_full_grads(cdsgd_plan *plan, const float *const *const *peer_grads)
{
    if (!plan) return CDSGD_ERR_NULL;
    const int np = plan->num_workers - 1;
    if (np == 0) return CDSGD_OK;  // a single worker's sum is its own gradient
    if (!peer_grads) return CDSGD_ERR_NULL;
    std::vector<const void *> image((size_t)plan->num_tensors * (size_t)np);
    for (int j = 0, slot = 0; j < plan->num_workers; ++j) {
        if (j == plan->self) continue;
        if (!peer_grads[j]) return CDSGD_ERR_NULL;
        for (int i = 0; i < plan->num_tensors; ++i) {
            if (!peer_grads[j][i]) return CDSGD_ERR_NULL;
            if (!aligned(peer_grads[j][i], 16)) return CDSGD_ERR_ALIGN;
            image[(size_t)i * (size_t)np + (size_t)slot] = peer_grads[j][i];
        }
        ++slot;
    }
    const size_t bytes = image.size() * sizeof(const void *);
    void *dev = plan->peer_grads_block;
    if (!dev && hipMalloc(&dev, bytes) != hipSuccess) {
        (void)hipGetLastError();
        return CDSGD_ERR_DEVICE;
    }
    if (hipMemcpy(dev, image.data(), bytes, hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipGetLastError();
        if (!plan->peer_grads_block) (void)hipFree(dev);
        return CDSGD_ERR_DEVICE;
    }
    plan->peer_grads_block = dev;
    plan->peer_grads = (const void **)dev;
    return CDSGD_OK;
}


int cdsgd_plan_set_thresholds(cdsgd_plan *plan, const float *thresholds)
{
    if (!plan) return CDSGD_ERR_NULL;
    bool all_pow2 = true;
    if (thresholds)
        for (int i = 0; i < plan->num_tensors; ++i) {
            if (!good_threshold(thresholds[i])) return CDSGD_ERR_PARAM;
            all_pow2 = all_pow2 && is_pow2_threshold(thresholds[i]);
        }
    std::vector<TensorDesc> next = plan->host_tensors;
    for (int i = 0; i < plan->num_tensors; ++i) next[(size_t)i].threshold = thresholds ? thresholds[i] : 0.0f;
    if (hipMemcpy(plan->tensors, next.data(), sizeof(TensorDesc) * next.size(), hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipGetLastError();
        return CDSGD_ERR_DEVICE;
    }
    plan->host_tensors.swap(next);
    plan->own_thresholds = thresholds != nullptr;
    plan->own_thresholds_pow2 = thresholds != nullptr && all_pow2;
    return CDSGD_OK;
}

size_t cdsgd_sparse_segments(size_t n) { return ((n + 15) / 16 + kSegWords - 1) / kSegWords; }

size_t cdsgd_sparse_words(size_t n) { return cdsgd_sparse_segments(n) * kSegStride; }

int cdsgd_sparse_encode(const uint32_t *packed, size_t n, uint32_t *sparse, uint32_t *segment_words,
                        void *hip_stream)
{
    if (!packed || !sparse) return CDSGD_ERR_NULL;
    if (n == 0 || cdsgd_sparse_segments(n) > kMaxGrid) return CDSGD_ERR_SIZE;
    if (!aligned(packed, 4) || !aligned(sparse, 4) || !aligned(segment_words, 4)) return CDSGD_ERR_ALIGN;
    const size_t pb = (size_t)packed_bytes_of(n), sb = cdsgd_sparse_words(n) * 4, cb = cdsgd_sparse_segments(n) * 4;
    if (overlap2(packed, pb, sparse, sb) || overlap2(packed, pb, segment_words, cb) ||
        overlap2(sparse, sb, segment_words, cb))
        return CDSGD_ERR_ALIAS;
    hipLaunchKernelGGL(k_sparse_encode, dim3((unsigned)cdsgd_sparse_segments(n)), dim3(256), 0,
                       (hipStream_t)hip_stream, packed, (unsigned long long)((n + 15) / 16), sparse, segment_words);
    return launch_status();
}

int cdsgd_decode_sum_sparse(const uint32_t *const *sparse, int num_workers, float *agg, size_t n, float threshold,
                            void *hip_stream)
{
    if (!sparse || !agg) return CDSGD_ERR_NULL;
    if (n == 0 || chunks_of(n) > kMaxGrid) return CDSGD_ERR_SIZE;
    if (!good_threshold(threshold)) return CDSGD_ERR_PARAM;
    if (num_workers < 1 || num_workers > CDSGD_MAX_WORKERS) return CDSGD_ERR_WORKERS;
    for (int j = 0; j < num_workers; ++j)
        if (!sparse[j]) return CDSGD_ERR_NULL;
    if (!aligned(agg, 16)) return CDSGD_ERR_ALIGN;
    for (int j = 0; j < num_workers; ++j)
        if (!aligned(sparse[j], 4)) return CDSGD_ERR_ALIGN;
    for (int j = 0; j < num_workers; ++j)
        if (overlap2(sparse[j], cdsgd_sparse_words(n) * 4, agg, n * sizeof(float))) return CDSGD_ERR_ALIAS;
    StreamTable tab;
    std::memset(&tab, 0, sizeof(tab));
    for (int j = 0; j < num_workers; ++j) tab.p[j] = reinterpret_cast<const uint8_t *>(sparse[j]);
    const unsigned grid = (unsigned)chunks_of(n);
    const float bias_t = -(2.0f * (float)num_workers) * threshold;
    if (is_pow2_threshold(threshold))
        hipLaunchKernelGGL((k_decode_sum_sparse<true, kSparseLanes>), dim3(grid), dim3(kSparseLanes), 0, (hipStream_t)hip_stream, tab,
                           num_workers, agg, extent_of(n), threshold, bias_t);
    else
        hipLaunchKernelGGL((k_decode_sum_sparse<false, kSparseLanes>), dim3(grid), dim3(kSparseLanes), 0, (hipStream_t)hip_stream, tab,
                           num_workers, agg, extent_of(n), threshold, bias_t);
    return launch_status();
}

int cdsgd_plan_set_peer_format(cdsgd_plan *plan, int format)
{
    if (!plan) return CDSGD_ERR_NULL;
    if (format != CDSGD_PEERS_PACKED && format != CDSGD_PEERS_SPARSE) return CDSGD_ERR_PARAM;
    plan->peers_sparse = format == CDSGD_PEERS_SPARSE;
    return CDSGD_OK;
}

int cdsgd_probe_streams(const float *const *reads, int num_reads, float *const *writes, int num_writes, size_t n,
                        float *sink, unsigned lds_bytes, void *hip_stream)
{
    if (num_reads < 0 || num_reads > kProbeMaxReads || num_writes < 0 || num_writes > kProbeMaxWrites ||
        num_reads + num_writes == 0 || lds_bytes > 65536u)
        return CDSGD_ERR_PARAM;
    if ((num_reads > 0 && !reads) || (num_writes > 0 && !writes) || (num_writes == 0 && !sink)) return CDSGD_ERR_NULL;
    if (n == 0 || n % 256 != 0 || n / 256 > 0xFFFFFFFFull / 64) return CDSGD_ERR_SIZE;
    ProbeStreams p;
    std::memset(&p, 0, sizeof(p));
    p.num_reads = num_reads;
    for (int i = 0; i < num_reads; ++i) {
        if (!reads[i]) return CDSGD_ERR_NULL;
        if (!aligned(reads[i], 16)) return CDSGD_ERR_ALIGN;
        p.r[i] = reads[i];
    }
    for (int i = 0; i < num_writes; ++i) {
        if (!writes[i]) return CDSGD_ERR_NULL;
        if (!aligned(writes[i], 16)) return CDSGD_ERR_ALIGN;
        for (int j = 0; j < num_reads; ++j)
            if (overlap(writes[i], reads[j], n * sizeof(float))) return CDSGD_ERR_ALIAS;
        for (int j = 0; j < i; ++j)
            if (overlap(writes[i], writes[j], n * sizeof(float))) return CDSGD_ERR_ALIAS;
        p.w[i] = writes[i];
    }
    const dim3 grid((unsigned)(n / 256)), block(64);
    hipStream_t s = (hipStream_t)hip_stream;
#define CDSGD_PROBE(R, W) hipLaunchKernelGGL((k_probe_streams<R, W>), grid, block, lds_bytes, s, p, sink)
    switch ((num_reads > 3 ? 4 : num_reads) * 4 + num_writes) {
    case 4 * 4 + 0: CDSGD_PROBE(-1, 0); break;
    case 4 * 4 + 1: CDSGD_PROBE(-1, 1); break;
    case 4 * 4 + 2: CDSGD_PROBE(-1, 2); break;
    case 4 * 4 + 3: CDSGD_PROBE(-1, 3); break;
    case 0 * 4 + 1: CDSGD_PROBE(0, 1); break;
    case 0 * 4 + 2: CDSGD_PROBE(0, 2); break;
    case 0 * 4 + 3: CDSGD_PROBE(0, 3); break;
    case 1 * 4 + 0: CDSGD_PROBE(1, 0); break;
    case 1 * 4 + 1: CDSGD_PROBE(1, 1); break;
    case 1 * 4 + 2: CDSGD_PROBE(1, 2); break;
    case 1 * 4 + 3: CDSGD_PROBE(1, 3); break;
    case 2 * 4 + 0: CDSGD_PROBE(2, 0); break;
    case 2 * 4 + 1: CDSGD_PROBE(2, 1); break;
    case 2 * 4 + 2: CDSGD_PROBE(2, 2); break;
    case 2 * 4 + 3: CDSGD_PROBE(2, 3); break;
    case 3 * 4 + 0: CDSGD_PROBE(3, 0); break;
    case 3 * 4 + 1: CDSGD_PROBE(3, 1); break;
    case 3 * 4 + 2: CDSGD_PROBE(3, 2); break;
    default: CDSGD_PROBE(3, 3); break;
    }
#undef CDSGD_PROBE
    return launch_status();
}

int cdsgd_plan_set_max_workgroups(cdsgd_plan *plan, int max_workgroups)
{
    if (!plan) return CDSGD_ERR_NULL;
    if (max_workgroups < 0) return CDSGD_ERR_PARAM;
    plan->max_workgroups = (unsigned)max_workgroups;
    return CDSGD_OK;
}

int cdsgd_step_warmup(cdsgd_plan *plan, long i, long warmup_steps, float lr_local, float lr_global,
                      void *hip_stream)
{
    if (!plan) return CDSGD_ERR_NULL;
    if (warmup_steps < 0 || i < 0 || i > warmup_steps || !std::isfinite(lr_local) || !std::isfinite(lr_global))
        return CDSGD_ERR_PARAM;
    const int mode = i == warmup_steps ? kLocalRule : (i == warmup_steps - 1 ? kLocalCopy : kLocalNone);
    return launch_full_pass(plan, mode, lr_local, lr_global, hip_stream);
}

int cdsgd_trainer_create(cdsgd_plan *plan, long warmup_steps, int k, float threshold, float lr_local,
                         float lr_global, cdsgd_trainer **out)
{
    if (!out) return CDSGD_ERR_NULL;
    *out = nullptr;
    if (!plan) return CDSGD_ERR_NULL;
    if (warmup_steps < 0 || k < 1 || !good_threshold(threshold) || !std::isfinite(lr_local) ||
        !std::isfinite(lr_global))
        return CDSGD_ERR_PARAM;
    cdsgd_trainer *t = new (std::nothrow) cdsgd_trainer;
    if (!t) return CDSGD_ERR_DEVICE;
    t->plan = plan;
    t->warmup_steps = warmup_steps;
    t->k = k;
    t->threshold = threshold;
    t->lr_local = lr_local;
    t->lr_global = lr_global;
    t->iteration = 0;
    *out = t;
    return CDSGD_OK;
}

int cdsgd_trainer_step(cdsgd_trainer *trainer, void *hip_stream, int *pass_kind)
{
    if (!trainer) return CDSGD_ERR_NULL;
    const long it = trainer->iteration;
    int rc, kind;
    if (it <= trainer->warmup_steps) {
        kind = CDSGD_PASS_WARMUP;
        rc = cdsgd_step_warmup(trainer->plan, it, trainer->warmup_steps, trainer->lr_local, trainer->lr_global,
                               hip_stream);
    } else {
        const long count = it - trainer->warmup_steps - 1;
        kind = (count % trainer->k) != 0 ? CDSGD_PASS_COMPRESSED : CDSGD_PASS_CORRECTION;
        rc = cdsgd_step_fused(trainer->plan, count, trainer->k, trainer->threshold, trainer->lr_local,
                              trainer->lr_global, hip_stream);
    }
    if (rc != CDSGD_OK) return rc;  // the iteration counter only advances on success
    trainer->iteration = it + 1;
    if (pass_kind) *pass_kind = kind;
    return CDSGD_OK;
}

long cdsgd_trainer_iteration(const cdsgd_trainer *trainer) { return trainer ? trainer->iteration : -1; }

int cdsgd_trainer_destroy(cdsgd_trainer *trainer)
{
    delete trainer;
    return CDSGD_OK;
}

}  // extern "C"

namespace {

std::mutex g_static_mutex;
constexpr int kStaticMaxDevices = 64;
unsigned char *g_static_ptr[kStaticMaxDevices] = {};

// Device address of `scratch` on the current device, looked up once per device.
int static_scratch(unsigned char **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kStaticMaxDevices) {
        (void)hipGetLastError();
        return CDSGD_ERR_DEVICE;
    }
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return CDSGD_ERR_DEVICE;
        }
        g_static_ptr[dev] = static_cast<unsigned char *>(p);
    }
    *out = g_static_ptr[dev];
    return CDSGD_OK;
}

// Streams host bytes into a region of the static array through kernel arguments:
// no host-to-device copy call, no staging memory, nothing a graph capture could not record.
struct StaticWriter {
    hipStream_t stream;
    unsigned char *dst;  // device address the next flush writes to
    StorePayload buf;
    unsigned fill = 0;
    bool ok = true;

    StaticWriter(hipStream_t s, unsigned char *d) : stream(s), dst(d) {}

    void flush()
    {
        if (fill == 0) return;
        while (fill % 16u) reinterpret_cast<unsigned char *>(&buf)[fill++] = 0;
        hipLaunchKernelGGL(k_static_store, dim3(1), dim3(256), 0, stream, buf, reinterpret_cast<uint4 *>(dst), fill / 16u);
        ok = ok && hipGetLastError() == hipSuccess;
        dst += fill;
        fill = 0;
    }

    void put(const void *src, unsigned bytes)
    {
        const unsigned char *p = static_cast<const unsigned char *>(src);
        while (bytes) {
            const unsigned take = bytes < kStorePayload - fill ? bytes : kStorePayload - fill;
            std::memcpy(reinterpret_cast<unsigned char *>(&buf) + fill, p, take);
            fill += take;
            p += take;
            bytes -= take;
            if (fill == kStorePayload) flush();
        }
    }
};

}  // namespace

extern "C" int cdsgd_step_fused_static(const cdsgd_tensor *tensors, int num_tensors,
                                       const uint32_t *const *const *peers, int num_workers, int self,
                                       int grad_dtype, long step, int k, float threshold, float lr_local,
                                       float lr_global, void *hip_stream)
{
    unsigned long long total_chunks = 0;
    bool all_agg = true;
    int rc = check_layer_list(tensors, num_tensors, peers, num_workers, self, grad_dtype, &total_chunks, &all_agg);
    if (rc != CDSGD_OK) return rc;
    if (!good_step_params(step, k, threshold, lr_local, lr_global)) return CDSGD_ERR_PARAM;
    if (num_tensors > kStaticMaxTensors || total_chunks > kStaticMaxChunks) return CDSGD_ERR_SIZE;
    const bool compressed = (step % k) != 0;
    if (!compressed && num_workers > 1 && !all_agg) return CDSGD_ERR_NULL;

    unsigned char *base = nullptr;
    rc = static_scratch(&base);
    if (rc != CDSGD_OK) return rc;
    hipStream_t s = (hipStream_t)hip_stream;
    const int num_peers = num_workers - 1;

    // descriptor table
    StaticWriter w(s, base + kStaticOffDesc);
    for (int i = 0; i < num_tensors; ++i) {
        const TensorDesc d = make_desc(tensors[i]);
        w.put(&d, sizeof(d));
    }
    w.flush();
    // chunk_start: running count of chunks, num_tensors + 1 entries
    w.dst = base + kStaticOffStart;
    unsigned start = 0;
    for (int i = 0; i < num_tensors; ++i) {
        w.put(&start, sizeof(start));
        start += (unsigned)chunks_of(tensors[i].n);
    }
    w.put(&start, sizeof(start));
    w.flush();
    // peers' streams, [tensor][peer], the own row left out (compressed passes only)
    if (compressed && num_peers > 0) {
        w.dst = base + kStaticOffPeers;
        for (int i = 0; i < num_tensors; ++i)
            for (int j = 0; j < num_workers; ++j) {
                if (j == self) continue;
                const uint8_t *ptr = reinterpret_cast<const uint8_t *>(peers[j][i]);
                w.put(&ptr, sizeof(ptr));
            }
        w.flush();
    }
    if (!w.ok) return CDSGD_ERR_DEVICE;
    // chunk table, on the device
    const unsigned total = (unsigned)total_chunks;
    hipLaunchKernelGGL(k_static_chunks, dim3((total + 255u) / 256u), dim3(256), 0, s,
                       reinterpret_cast<const unsigned *>(base + kStaticOffStart), num_tensors,
                       reinterpret_cast<ChunkRef *>(base + kStaticOffChunks), total);
    if (hipGetLastError() != hipSuccess) return CDSGD_ERR_DEVICE;

    PlanTables pt;
    pt.tensors = reinterpret_cast<TensorDesc *>(base + kStaticOffDesc);
    pt.chunks = reinterpret_cast<ChunkRef *>(base + kStaticOffChunks);
    pt.peers = reinterpret_cast<const uint8_t **>(base + kStaticOffPeers);
    pt.num_tensors = num_tensors;
    pt.num_workers = num_workers;
    pt.self = self;
    pt.num_chunks = total;
    pt.has_agg_full = all_agg;
    pt.grad_type = grad_dtype;
    return launch_formal_pass(&pt, step, k, threshold, lr_local, lr_global, true, hip_stream);
}
