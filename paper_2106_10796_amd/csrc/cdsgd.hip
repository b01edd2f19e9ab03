// CD-SGD per-step data-parallel hot path for gfx950 (MI355X): kernels and C ABI.
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
//   * Of the single-tensor kernels, decode-and-sum and the update give a chunk
//     to a workgroup of kBlock lanes, lane `tid` taking quads j*kBlock + tid;
//     quantise-and-pack works in single-wave pieces.
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

// Launch shapes and cache policy are chosen by measurement on MI355X; each kernel
// states its own.  CDSGD_BLOCK x CDSGD_QPL is the shape of the chunk-per-workgroup
// kernels (k_decode_sum, k_update) and fixes the chunk size of the plan tables.
// Non-temporal loads and stores are worth about 15 % (every byte is touched once
// per step, so nothing should stay in L2 or the memory-side cache).
#ifndef CDSGD_BLOCK
#define CDSGD_BLOCK 512
#endif
#ifndef CDSGD_QPL
#define CDSGD_QPL 2
#endif
#ifndef CDSGD_NT
#define CDSGD_NT 1
#endif
#ifndef CDSGD_NT_LOAD
#define CDSGD_NT_LOAD CDSGD_NT
#endif
#ifndef CDSGD_NT_STORE
#define CDSGD_NT_STORE CDSGD_NT
#endif
#ifndef CDSGD_NT_CODES
#define CDSGD_NT_CODES 0
#endif
#ifndef CDSGD_XCD_FULL
#define CDSGD_XCD_FULL 0
#endif
#ifndef CDSGD_PIECE_WAVES
#define CDSGD_PIECE_WAVES 4
#endif
#ifndef CDSGD_FEW_PEERS
#define CDSGD_FEW_PEERS 8
#endif
#ifndef CDSGD_XCD_PIECES
#define CDSGD_XCD_PIECES 1
#endif
#ifndef CDSGD_FULL_BLOCK
#define CDSGD_FULL_BLOCK 64
#endif
#ifndef CDSGD_PEER_BATCH
#define CDSGD_PEER_BATCH 4
#endif

namespace {

constexpr unsigned kBlock = CDSGD_BLOCK;          // lanes per workgroup
constexpr unsigned kQpl = CDSGD_QPL;              // quads per lane
constexpr unsigned kChunkQuads = kBlock * kQpl;   // quads (= packed bytes) per chunk
constexpr unsigned kChunkElems = kChunkQuads * 4; // elements per chunk
constexpr int kPeerBatch = CDSGD_PEER_BATCH;      // peers whose bytes are in flight together
static_assert(kQpl == 1 || kQpl == 2 || kQpl == 4, "a lane's packed bytes must fit one register");
static_assert(CDSGD_GRAD_F32 == 0 && CDSGD_GRAD_BF16 == 1 && CDSGD_GRAD_F16 == 2, "header and kernels agree");

typedef float f4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------
// 128-bit loads / stores, with the ragged end of a tensor handled per element
// ---------------------------------------------------------------------------
__device__ __forceinline__ f4 ld4(const float *base, unsigned qi)
{
    const f4 *p = reinterpret_cast<const f4 *>(base) + qi;
#if CDSGD_NT_LOAD
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}

__device__ __forceinline__ void st4(float *base, unsigned qi, f4 v)
{
    f4 *p = reinterpret_cast<f4 *>(base) + qi;
#if CDSGD_NT_STORE
    __builtin_nontemporal_store(v, p);
#else
    *p = v;
#endif
}

// cnt = number of elements of this quad that exist (4 in the interior).
template <bool G>
__device__ __forceinline__ f4 ld4g(const float *base, unsigned qi, int cnt)
{
    if (!G || cnt == 4) return ld4(base, qi);
    f4 v = {0.0f, 0.0f, 0.0f, 0.0f};
    const float *p = base + 4u * qi;
    if (cnt > 0) v.x = p[0];
    if (cnt > 1) v.y = p[1];
    if (cnt > 2) v.z = p[2];
    return v;
}

template <bool G>
__device__ __forceinline__ void st4g(float *base, unsigned qi, int cnt, f4 v)
{
    if (!G || cnt == 4) {
        st4(base, qi, v);
        return;
    }
    float *p = base + 4u * qi;
    if (cnt > 0) p[0] = v.x;
    if (cnt > 1) p[1] = v.y;
    if (cnt > 2) p[2] = v.z;
}

// Gradient element types: fp32, or bf16 / fp16 widened exactly to fp32 on load
// (everything downstream of the load is the fp32 path).
constexpr int kGradF32 = 0, kGradBF16 = 1, kGradF16 = 2;

template <int GT>
__device__ __forceinline__ constexpr unsigned grad_bytes()
{
    return GT == kGradF32 ? 4u : 2u;
}

typedef unsigned u2 __attribute__((ext_vector_type(2)));

template <int GT>
__device__ __forceinline__ float widen16(unsigned h)  // h: the 16-bit pattern in the low half
{
    if (GT == kGradBF16) return __builtin_bit_cast(float, h << 16);
    return (float)__builtin_bit_cast(_Float16, (unsigned short)h);
}

// One quad of a gradient buffer; `base` is the chunk's first element.
template <bool G, int GT>
__device__ __forceinline__ f4 ldgrad(const void *base, unsigned qi, int cnt)
{
    if (GT == kGradF32) return ld4g<G>(static_cast<const float *>(base), qi, cnt);
    if (!G || cnt == 4) {
        const u2 *p = static_cast<const u2 *>(base) + qi;
#if CDSGD_NT_LOAD
        const u2 v = __builtin_nontemporal_load(p);
#else
        const u2 v = *p;
#endif
        return f4{widen16<GT>(v.x & 0xFFFFu), widen16<GT>(v.x >> 16), widen16<GT>(v.y & 0xFFFFu),
                  widen16<GT>(v.y >> 16)};
    }
    f4 v = {0.0f, 0.0f, 0.0f, 0.0f};
    const unsigned short *p = static_cast<const unsigned short *>(base) + 4u * qi;
    if (cnt > 0) v.x = widen16<GT>(p[0]);
    if (cnt > 1) v.y = widen16<GT>(p[1]);
    if (cnt > 2) v.z = widen16<GT>(p[2]);
    return v;
}

template <int GT>
__device__ __forceinline__ const void *grad_at(const void *grad, size_t quad0)
{
    return static_cast<const char *>(grad) + quad0 * (4u * grad_bytes<GT>());
}

template <bool G>
__device__ __forceinline__ int quad_count(unsigned rem_elems, unsigned qi)
{
    if (!G) return 4;
    int c = (int)rem_elems - (int)(4u * qi);
    return c < 0 ? 0 : (c > 4 ? 4 : c);
}

// ---------------------------------------------------------------------------
// a1 + a2: error-feedback threshold quantiser (Sec. 2.3, Sec. 3.4.1)
// ---------------------------------------------------------------------------
// a = r + g; |a| >= t sends sign(a)*t and keeps the rest.  `sent` is what the
// code stands for (+t, -t or +0); a - sent is bit-identical to a - t, a + t and
// a in the three cases.  Returns the 2-bit code (1 = +t, 2 = -t).
__device__ __forceinline__ unsigned quantize1(float g, float &r, float t, float &sent)
{
    const float a = r + g;
    const bool pos = a >= t;
    const bool neg = a <= -t;
    sent = pos ? t : (neg ? -t : 0.0f);
    r = a - sent;
    return pos ? 1u : (neg ? 2u : 0u);
}

// One quad: residual updated in place, returns the packed byte.
__device__ __forceinline__ unsigned quantize_quad(const f4 g, f4 &r, float t, f4 &sent)
{
    float s0, s1, s2, s3, r0 = r.x, r1 = r.y, r2 = r.z, r3 = r.w;
    const unsigned c0 = quantize1(g.x, r0, t, s0);
    const unsigned c1 = quantize1(g.y, r1, t, s1);
    const unsigned c2 = quantize1(g.z, r2, t, s2);
    const unsigned c3 = quantize1(g.w, r3, t, s3);
    r = f4{r0, r1, r2, r3};
    sent = f4{s0, s1, s2, s3};
    return c0 | (c1 << 2) | (c2 << 4) | (c3 << 6);
}

// ---------------------------------------------------------------------------
// a4: decode-and-sum (Sec. 3.2.1; sum of eq. 10)
// ---------------------------------------------------------------------------
// A lane keeps the packed bytes of its kQpl quads of one worker in one
// register: byte j = quad j.

// Bytes of one worker for this lane's quads.
template <bool G>
__device__ __forceinline__ unsigned load_codes(const uint8_t *stream, unsigned tid, unsigned rem_bytes)
{
    unsigned w = 0;
#pragma unroll
    for (unsigned j = 0; j < kQpl; ++j) {
        const unsigned qi = j * kBlock + tid;
        unsigned b = 0;
#if CDSGD_NT_CODES
        if (!G || qi < rem_bytes) b = __builtin_nontemporal_load(stream + qi);
#else
        if (!G || qi < rem_bytes) b = stream[qi];
#endif
        w |= b << (8 * j);
    }
    return w;
}

// Literal fp32 chain: agg += value(code) for the 4*kQpl elements of this lane,
// one rounded add per element.  The codes are first rewritten, 16 at a time,
// as 2-bit two's-complement counts (01 -> +1, 10 -> -1, 00 and 11 -> 0) so
// that one signed bit-field extract yields the multiplier.
__device__ __forceinline__ void chain_codes(f4 (&agg)[kQpl], unsigned w, float t)
{
    const unsigned x = w & 0x55555555u;
    const unsigned y = (w >> 1) & 0x55555555u;
    const unsigned lo = x ^ y;
    const unsigned hi = y & ~x;
    const unsigned s = lo | (hi << 1);
#pragma unroll
    for (unsigned j = 0; j < kQpl; ++j) {
#pragma unroll
        for (unsigned c = 0; c < 4; ++c) {
            const int m = ((int)(s << (30u - (8u * j + 2u * c)))) >> 30;
            agg[j][c] = __builtin_fmaf((float)m, t, agg[j][c]);
        }
    }
}

// Count form for thresholds that are powers of two (every partial sum of the
// chain is then exact, so sum == count * t bit for bit).  Per worker the 16
// codes become biased counts (2 + value) in 2-bit fields without borrows, and
// are added into four registers of byte-wide fields: acc[c] byte j belongs to
// element c of quad j.
__device__ __forceinline__ void count_codes(unsigned (&acc)[4], unsigned w)
{
    const unsigned z = ((w & 0x55555555u) | 0xAAAAAAAAu) - ((w >> 1) & 0x55555555u);
    acc[0] += z & 0x03030303u;
    acc[1] += (z >> 2) & 0x03030303u;
    acc[2] += (z >> 4) & 0x03030303u;
    acc[3] += (z >> 6) & 0x03030303u;
}

// acc holds 2*num_summed + sum of values; bias_t = -(2*num_summed)*t.
__device__ __forceinline__ void counts_to_sum(f4 (&agg)[kQpl], const unsigned (&acc)[4], float t,
                                              float bias_t)
{
#pragma unroll
    for (unsigned j = 0; j < kQpl; ++j) {
#pragma unroll
        for (unsigned c = 0; c < 4; ++c) {
            const float cnt = (float)((acc[c] >> (8u * j)) & 0xFFu);
            agg[j][c] = __builtin_fmaf(cnt, t, bias_t);
        }
    }
}

// Sum workers [p_begin, p_end) of a pointer table into agg (chain) or acc (count),
// kPeerBatch streams in flight at a time.
template <bool G, bool POW2>
__device__ __forceinline__ void sum_streams(f4 (&agg)[kQpl], unsigned (&acc)[4],
                                            const uint8_t *const *__restrict__ tab, int p_begin,
                                            int p_end, size_t quad0, unsigned tid,
                                            unsigned rem_bytes, float t)
{
    int p = p_begin;
    for (; p + kPeerBatch <= p_end; p += kPeerBatch) {
        unsigned w[kPeerBatch];
#pragma unroll
        for (int i = 0; i < kPeerBatch; ++i) w[i] = load_codes<G>(tab[p + i] + quad0, tid, rem_bytes);
#pragma unroll
        for (int i = 0; i < kPeerBatch; ++i) {
            if (POW2) count_codes(acc, w[i]);
            else chain_codes(agg, w[i], t);
        }
    }
    if (kPeerBatch > 4 && p + 4 <= p_end) {
        unsigned w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = load_codes<G>(tab[p + i] + quad0, tid, rem_bytes);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (POW2) count_codes(acc, w[i]);
            else chain_codes(agg, w[i], t);
        }
        p += 4;
    }
    for (; p < p_end; ++p) {
        const unsigned w = load_codes<G>(tab[p] + quad0, tid, rem_bytes);
        if (POW2) count_codes(acc, w);
        else chain_codes(agg, w, t);
    }
}

// ---------------------------------------------------------------------------
// device-side tables of a plan
// ---------------------------------------------------------------------------
// How a tensor of n elements splits into chunks: `full_chunks` chunks hold
// kChunkElems elements each; if anything is left, one more chunk holds the
// ragged end: tail_elems elements (< kChunkElems) and tail_bytes bytes of the
// packed stream (the bytes of the last word past the last element included).
// Everything is 32-bit and uniform, so the interior/tail decision is a scalar
// compare on the chunk number.
struct Extent {
    unsigned full_chunks;
    unsigned tail_elems;
    unsigned tail_bytes;
    unsigned pad_;
};

struct TensorDesc {
    float *w_global;
    float *w_local;
    float *residual;
    const void *grad;  // fp32, bf16 or fp16 (the plan's gradient type)
    uint8_t *packed_self;
    const float *agg_full;
    Extent ext;
    float threshold;  // > 0: this tensor's own threshold (cdsgd_plan_set_thresholds); 0: the call's
    unsigned pad_;
};

struct ChunkRef {
    unsigned tensor;  // index into the TensorDesc table
    unsigned chunk;   // chunk number inside that tensor
};

// Every kernel over a layer list walks the pieces of the chunk table from its workgroup number
// in steps of the grid size.  Normally the grid has one workgroup per piece and the loop runs
// once; a plan with a workgroup limit (cdsgd_plan_set_max_workgroups) launches fewer
// workgroups, which then take several pieces each and leave compute units free for other
// kernels.  How pieces are dealt to the 8 XCDs is piece_of_workgroup's business.

// ---------------------------------------------------------------------------
// kernels
// ---------------------------------------------------------------------------

// a4 for one tensor; the worker pointers travel in the kernel arguments.
struct StreamTable {
    const uint8_t *p[CDSGD_MAX_WORKERS];
};

template <bool G, bool POW2>
__device__ __forceinline__ void decode_sum_chunk(const StreamTable &tab, int num_workers,
                                                 float *__restrict__ agg_out, size_t quad0,
                                                 unsigned rem_elems, unsigned rem_bytes, float t,
                                                 float bias_t)
{
    const unsigned tid = threadIdx.x;
    f4 agg[kQpl];
    unsigned acc[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (unsigned j = 0; j < kQpl; ++j) agg[j] = f4{0.0f, 0.0f, 0.0f, 0.0f};
    sum_streams<G, POW2>(agg, acc, tab.p, 0, num_workers, quad0, tid, rem_bytes, t);
    if (POW2) counts_to_sum(agg, acc, t, bias_t);
#pragma unroll
    for (unsigned j = 0; j < kQpl; ++j) {
        const unsigned qi = j * kBlock + tid;
        st4g<G>(agg_out, qi, quad_count<G>(rem_elems, qi), agg[j]);
    }
}

template <bool POW2>
__global__ __launch_bounds__(CDSGD_BLOCK) void k_decode_sum(StreamTable tab, int num_workers,
                                                            float *__restrict__ agg, Extent ext, float t,
                                                            float bias_t)
{
    const unsigned chunk = blockIdx.x;
    const size_t quad0 = (size_t)chunk * kChunkQuads;
    agg += 4 * quad0;
    if (chunk < ext.full_chunks)
        decode_sum_chunk<false, POW2>(tab, num_workers, agg, quad0, kChunkElems, kChunkQuads, t, bias_t);
    else
        decode_sum_chunk<true, POW2>(tab, num_workers, agg, quad0, ext.tail_elems, ext.tail_bytes, t, bias_t);
}

// a5 + a6 (eq. 10, eq. 11), both from the weight that was loaded.
template <bool G, bool LOCAL, bool GLOBAL, int GT = kGradF32>
__device__ __forceinline__ void update_chunk(float *__restrict__ wg, float *__restrict__ wl,
                                             const void *__restrict__ grad,
                                             const float *__restrict__ agg, unsigned rem_elems,
                                             float lr_local, float scale)
{
    const unsigned tid = threadIdx.x;
    f4 w[kQpl], g[kQpl], a[kQpl];
    int cnt[kQpl];
#pragma unroll
    for (unsigned j = 0; j < kQpl; ++j) {
        const unsigned qi = j * kBlock + tid;
        cnt[j] = quad_count<G>(rem_elems, qi);
        w[j] = ld4g<G>(wg, qi, cnt[j]);
        if (LOCAL) g[j] = ldgrad<G, GT>(grad, qi, cnt[j]);
        if (GLOBAL) a[j] = ld4g<G>(agg, qi, cnt[j]);
    }
#pragma unroll
    for (unsigned j = 0; j < kQpl; ++j) {
        const unsigned qi = j * kBlock + tid;
        if (LOCAL) {
            f4 v;
#pragma unroll
            for (unsigned c = 0; c < 4; ++c) v[c] = __builtin_fmaf(-lr_local, g[j][c], w[j][c]);
            st4g<G>(wl, qi, cnt[j], v);
        }
        if (GLOBAL) {
            f4 v;
#pragma unroll
            for (unsigned c = 0; c < 4; ++c) v[c] = __builtin_fmaf(-scale, a[j][c], w[j][c]);
            st4g<G>(wg, qi, cnt[j], v);
        }
    }
}

template <bool LOCAL, bool GLOBAL>
__global__ __launch_bounds__(CDSGD_BLOCK) void k_update(float *__restrict__ wg, float *__restrict__ wl,
                                                        const float *__restrict__ grad,
                                                        const float *__restrict__ agg, Extent ext,
                                                        float lr_local, float scale)
{
    const unsigned chunk = blockIdx.x;
    const size_t quad0 = (size_t)chunk * kChunkQuads;
    wg += 4 * quad0;
    if (LOCAL) {
        wl += 4 * quad0;
        grad += 4 * quad0;
    }
    if (GLOBAL) agg += 4 * quad0;
    if (chunk < ext.full_chunks) update_chunk<false, LOCAL, GLOBAL>(wg, wl, grad, agg, kChunkElems, lr_local, scale);
    else update_chunk<true, LOCAL, GLOBAL>(wg, wl, grad, agg, ext.tail_elems, lr_local, scale);
}

typedef unsigned u4 __attribute__((ext_vector_type(4)));

// values of the codes of a register, as 2-bit two's-complement fields (01 -> +1, 10 -> -1, else 0)
__device__ __forceinline__ unsigned signed_fields(unsigned w)
{
    const unsigned x = w & 0x55555555u;
    const unsigned y = (w >> 1) & 0x55555555u;
    return (x ^ y) | ((y & ~x) << 1);
}

// ---------------------------------------------------------------------------
// Sparse form of a packed stream (this library's own wire format, see cdsgd.h)
// ---------------------------------------------------------------------------
// A segment is the 256 packed words of one chunk: 8 bitmap words (bit b of word m set iff packed
// word 32 m + b of the segment is non-zero), then the non-zero words in index order.  Segments
// sit at a fixed stride of 264 words.
constexpr unsigned kSegWords = 256;
constexpr unsigned kSegStride = 8 + kSegWords;
static_assert(kChunkQuads == 4 * kSegWords, "a segment of the sparse form is the packed stream of one chunk");

// Packed words w0 .. w0+3 (w0 a multiple of 4) of a segment whose 8 bitmap words are in `bitmap`
// (LDS).  The non-zero ones among them lie next to each other behind the bitmap, so one 128-bit
// load fetches them (it may run into slots behind the segment's last value, never past its 264
// words); the bitmap says which of the four each loaded word is.
__device__ __forceinline__ u4 sparse_words4(const uint32_t *__restrict__ seg, const uint32_t *bitmap, unsigned w0)
{
    const unsigned m = w0 >> 5;
    unsigned before = 0;  // non-zero words of the segment in front of bitmap word m
#pragma unroll
    for (unsigned x = 0; x < 8; ++x)
        if (x < m) before += (unsigned)__builtin_popcount(bitmap[x]);
    const unsigned bm = bitmap[m];
    const unsigned bit = w0 & 31u;
    const unsigned four = (bm >> bit) & 15u;
    u4 out = {0u, 0u, 0u, 0u};
    if (four != 0u) {
        typedef unsigned u4a __attribute__((ext_vector_type(4), aligned(4)));
        const unsigned pos = 8u + before + (unsigned)__builtin_popcount(bm & ((1u << bit) - 1u));
        const u4 v = *reinterpret_cast<const u4a *>(seg + pos);
        unsigned rank = 0;
#pragma unroll
        for (unsigned i = 0; i < 4; ++i)
            if ((four >> i) & 1u) {
                out[i] = rank == 0 ? v[0] : (rank == 1 ? v[1] : (rank == 2 ? v[2] : v[3]));
                ++rank;
            }
    }
    return out;
}

// One workgroup of 256 lanes per segment: lane i owns packed word i.
__global__ __launch_bounds__(256) void k_sparse_encode(const uint32_t *__restrict__ packed, unsigned long long nw,
                                                       uint32_t *__restrict__ sparse,
                                                       uint32_t *__restrict__ seg_words)
{
    __shared__ unsigned wave_count[4];
    const unsigned i = threadIdx.x, wave = i >> 6, lane = i & 63u;
    const unsigned long long w = (unsigned long long)blockIdx.x * kSegWords + i;
    const uint32_t v = w < nw ? packed[w] : 0u;
    const unsigned long long mask = __ballot(v != 0u);  // the wave's 64 words: two bitmap words
    if (lane == 0) wave_count[wave] = (unsigned)__builtin_popcountll(mask);
    __syncthreads();
    unsigned before = 0, total = 0;
#pragma unroll
    for (unsigned x = 0; x < 4; ++x) {
        if (x < wave) before += wave_count[x];
        total += wave_count[x];
    }
    uint32_t *seg = sparse + (size_t)blockIdx.x * kSegStride;
    if (lane == 0) {
        seg[2 * wave] = (uint32_t)mask;
        seg[2 * wave + 1] = (uint32_t)(mask >> 32);
    }
    if (v != 0u) seg[8u + before + (unsigned)__builtin_popcountll(mask & ((1ull << lane) - 1ull))] = v;
    if (i == 0 && seg_words) seg_words[blockIdx.x] = 8u + total;
}

// a4 on sparse streams, one tensor: 512 lanes per chunk, lane tid takes quads tid and 512 + tid.
// Four workers at a time are rebuilt into LDS (lane i < 256 rebuilds packed word i of each), then
// every lane picks its two bytes of each.
template <bool POW2>
__global__ __launch_bounds__(512) void k_decode_sum_sparse(StreamTable tab, int num_workers,
                                                           float *__restrict__ agg_out, Extent ext, float t,
                                                           float bias_t)
{
    __shared__ uint32_t words[4][kSegWords];
    const unsigned tid = threadIdx.x;
    const unsigned chunk = blockIdx.x;
    const bool tail = chunk >= ext.full_chunks;
    const unsigned rem_elems = tail ? ext.tail_elems : kChunkElems;
    f4 agg[2] = {f4{0.0f, 0.0f, 0.0f, 0.0f}, f4{0.0f, 0.0f, 0.0f, 0.0f}};
    unsigned acc[4] = {0u, 0u, 0u, 0u};
    for (int p0 = 0; p0 < num_workers; p0 += 4) {
        const int np = num_workers - p0 < 4 ? num_workers - p0 : 4;
        if (tid < kSegWords) {
            for (int k = 0; k < np; ++k) {
                const uint32_t *seg = reinterpret_cast<const uint32_t *>(tab.p[p0 + k]) + (size_t)chunk * kSegStride;
                const unsigned m = tid >> 5, bit = tid & 31u;
                const unsigned bm = seg[m];
                uint32_t v = 0u;
                if ((bm >> bit) & 1u) {
                    unsigned before = 0;
                    for (unsigned x = 0; x < m; ++x) before += (unsigned)__builtin_popcount(seg[x]);
                    v = seg[8u + before + (unsigned)__builtin_popcount(bm & ((1u << bit) - 1u))];
                }
                words[k][tid] = v;
            }
        }
        __syncthreads();
        for (int k = 0; k < np; ++k) {
            const uint8_t *bytes = reinterpret_cast<const uint8_t *>(words[k]);
            const unsigned w = (unsigned)bytes[tid] | ((unsigned)bytes[512u + tid] << 8);
            if (POW2) {
                const unsigned z = ((w & 0x55555555u) | 0xAAAAAAAAu) - ((w >> 1) & 0x55555555u);
                acc[0] += z & 0x03030303u;
                acc[1] += (z >> 2) & 0x03030303u;
                acc[2] += (z >> 4) & 0x03030303u;
                acc[3] += (z >> 6) & 0x03030303u;
            } else {
                const unsigned sf = signed_fields(w);
#pragma unroll
                for (unsigned j = 0; j < 2; ++j)
#pragma unroll
                    for (unsigned c = 0; c < 4; ++c) {
                        const int mlt = ((int)(sf << (30u - (8u * j + 2u * c)))) >> 30;
                        agg[j][c] = __builtin_fmaf((float)mlt, t, agg[j][c]);
                    }
            }
        }
        __syncthreads();
    }
    float *out = agg_out + (size_t)chunk * kChunkElems;
#pragma unroll
    for (unsigned j = 0; j < 2; ++j) {
        const unsigned qi = j * 512u + tid;
        if (POW2) {
#pragma unroll
            for (unsigned c = 0; c < 4; ++c)
                agg[j][c] = __builtin_fmaf((float)((acc[c] >> (8u * j)) & 0xFFu), t, bias_t);
        }
        int cnt = (int)rem_elems - (int)(4u * qi);
        cnt = cnt < 0 ? 0 : (cnt > 4 ? 4 : cnt);
        if (cnt == 4) st4(out, qi, agg[j]);
        else st4g<true>(out, qi, cnt, agg[j]);
    }
}

// a1-a3 for one tensor, one wave per piece of L = 64 quads (measured: 6.68 TB/s against 6.41 TB/s for
// 512-lane workgroups with two quads per lane; the other two single-tensor kernels are faster in that
// shape and keep it).  `ext` describes the tensor in pieces: full_chunks whole pieces, then at most one
// ragged piece of tail_elems elements and tail_bytes packed bytes.
template <unsigned L>
__global__ __launch_bounds__(L) void k_quantize_pack(const float *__restrict__ grad, float *__restrict__ resid,
                                                       uint8_t *__restrict__ packed, Extent ext, float t)
{
    const unsigned piece = blockIdx.x, lane = threadIdx.x;
    const size_t quad0 = (size_t)piece * L;
    grad += 4 * quad0;
    resid += 4 * quad0;
    packed += quad0;
    f4 sent;
    if (piece < ext.full_chunks) {
        const f4 g = ld4(grad, lane);
        f4 r = ld4(resid, lane);
        const unsigned b = quantize_quad(g, r, t, sent);
        st4(resid, lane, r);
        packed[lane] = (uint8_t)b;
    } else {
        const int cnt = quad_count<true>(ext.tail_elems, lane);
        const f4 g = ld4g<true>(grad, lane, cnt);
        f4 r = ld4g<true>(resid, lane, cnt);
        const unsigned b = quantize_quad(g, r, t, sent);
        st4g<true>(resid, lane, cnt, r);
        if (lane < ext.tail_bytes) packed[lane] = (uint8_t)b;
    }
}

// ---------------------------------------------------------------------------
// Measurement aid: bare streaming with a given mix of read and write streams
// ---------------------------------------------------------------------------
// One wave per 64-quad piece, non-temporal 128-bit loads and stores, no arithmetic beyond adding
// what was read: what the memory system gives a kernel that moves R + W streams the way the fused
// kernels move theirs.  With W == 0 the sum goes to `sink` only if it has a value it cannot have.
constexpr int kProbeMaxReads = 17, kProbeMaxWrites = 3;
struct ProbeStreams {
    const float *r[kProbeMaxReads];
    float *w[kProbeMaxWrites];
    int num_reads;
};

// R >= 0: that many read streams, all loads in flight at once.  R < 0: p.num_reads streams, one
// load in flight per lane (the order the correction pass reads the workers' gradients in).
template <int R, int W>
__global__ __launch_bounds__(64) void k_probe_streams(ProbeStreams p, float *sink)
{
    const size_t quad0 = (size_t)blockIdx.x * 64u;
    const unsigned lane = threadIdx.x;
    f4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
    if (R >= 0) {
        f4 v[R > 0 ? R : 1];
#pragma unroll
        for (int i = 0; i < R; ++i) v[i] = ld4(p.r[i] + 4 * quad0, lane);
#pragma unroll
        for (int i = 0; i < R; ++i) acc = acc + v[i];
    } else {
        for (int i = 0; i < p.num_reads; ++i) acc = acc + ld4(p.r[i] + 4 * quad0, lane);
    }
#pragma unroll
    for (int i = 0; i < W; ++i) st4(p.w[i] + 4 * quad0, lane, acc + (float)i);
    if (W == 0) {
        const float s = acc.x + acc.y + acc.z + acc.w;
        if (s == -1.2345678e30f) sink[blockIdx.x] = s;
    }
}

// Piece-granular kernels: which piece workgroup b takes.  Workgroup b runs on XCD b % 8.  Within
// a block of 8 chunks' worth of workgroups, XCD k takes every piece of chunk k, so that the two
// halves of a 128-byte line of a peer's codes, and the pieces' reads of the chunk's table
// entries, meet in one L2 (measured on the ResNet-50-shaped list: 6.1 -> 6.8 TB/s).  The last,
// incomplete block keeps the plain order.  A bijection on [0, num_pieces) for any grid size.
template <bool XCD>
__device__ __forceinline__ unsigned long long piece_of_workgroup(unsigned long long b, unsigned per_chunk,
                                                                 unsigned long long num_pieces)
{
    if (!XCD) return b;
#if CDSGD_XCD_PIECES
    const unsigned long long group = 8ull * per_chunk;
    const unsigned long long blk = b / group, within = b % group;
    if ((blk + 1) * group <= num_pieces) return (blk * 8 + within % 8) * per_chunk + within / 8;
#endif
    return b;
}

// ---------------------------------------------------------------------------
// Fused compressed step (a1-a6), one workgroup per piece of a chunk
// ---------------------------------------------------------------------------
// A piece is 256 quads (1024 elements): 4 KiB of every fp32 stream and 256 bytes, two whole
// 128-byte lines, of every packed stream.  Its workgroup has 256 lanes (four waves), one quad
// and therefore one packed byte per lane.
//
// The peers' codes of a piece are fetched with ONE 128-bit load instruction per 16 peers: lane L
// takes bytes [16 (L % 16), +16) of peer L / 16, the workgroup writes them to LDS as
// [peer][byte], and every lane then reads its own byte of each peer back (LDS staging instead
// of one byte-wide global load per peer and lane).  No load of a peer's codes depends on
// another, so a workgroup's life is one round trip to memory however many workers there are,
// and the memory system sees the packed streams as whole lines.
//
// Measured on the VGG-16-shaped list (N = 16, count form): 6.3-6.4 TB/s, where 512-lane
// workgroups that took a whole chunk, two quads per lane and a byte load per peer, reached
// 6.0 TB/s; with one wave per piece (64 bytes per peer, half a line) 5.8-6.0 TB/s.
// Waves per piece: four for many workers (two whole lines of every packed stream per workgroup),
// one for few (N <= 9: the fp32 streams dominate, and they run best in single-wave workgroups).
constexpr unsigned kPieceWavesMany = CDSGD_PIECE_WAVES;
constexpr int kFewPeers = CDSGD_FEW_PEERS;
constexpr unsigned kPeerSlots = 64;  // LDS rows: peers rounded up to a multiple of 16 (63 peers at most)
static_assert(CDSGD_MAX_WORKERS - 1 <= kPeerSlots, "an LDS row for every peer");
static_assert(kChunkQuads % (64 * kPieceWavesMany) == 0, "pieces tile a chunk");

template <unsigned kPieceWaves, bool G, bool POW2, bool WRITE_LOCAL, int GT, bool SPARSE>
__device__ __forceinline__ void fused_piece(const TensorDesc &d, const uint8_t *const *__restrict__ peers,
                                            int num_peers, int self, size_t quad0, unsigned piece,
                                            unsigned rem_elems, unsigned rem_bytes, float t, float lr_local,
                                            float scale, uint8_t *lds)
{
    constexpr unsigned kPieceQuads = 64 * kPieceWaves;  // lanes per workgroup, one quad each
    const unsigned lane = threadIdx.x;
    const unsigned qi = piece * kPieceQuads + lane;  // quad of the chunk = byte of the chunk's packed streams
    const void *__restrict__ grad = grad_at<GT>(d.grad, quad0);
    float *__restrict__ resid = d.residual + 4 * quad0;
    float *__restrict__ wg = d.w_global + 4 * quad0;
    float *__restrict__ wl = d.w_local + 4 * quad0;
    uint8_t *__restrict__ pself = d.packed_self + quad0;
    const int cnt = quad_count<G>(rem_elems, qi);

    // the peers' bytes of this piece: 16 peers per load instruction
    constexpr unsigned kParts = kPieceQuads / 16;        // 16-byte parts of a peer's bytes of one piece
    const unsigned part = lane % kParts;                 // which of them this lane fetches
    const unsigned first = piece * kPieceQuads + 16u * part;  // its first byte within the chunk
    const int groups = (num_peers + 15) >> 4;
    uint32_t *bitmaps = reinterpret_cast<uint32_t *>(lds + kPeerSlots * kPieceQuads);  // [peer][8], sparse form only
    if (SPARSE) {
        // the segments' bitmaps first (8 words per peer, one word per lane), through LDS to every lane
        for (unsigned e = lane; e < 8u * 16u * (unsigned)groups; e += kPieceQuads) {
            const int p = (int)(e >> 3);
            bitmaps[e] = p < num_peers ? (reinterpret_cast<const uint32_t *>(peers[p]) +
                                          (quad0 / kChunkQuads) * kSegStride)[e & 7u]
                                       : 0u;
        }
        if (kPieceWaves == 1) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        } else {
            __syncthreads();
        }
    }
    u4 cw[kPeerSlots / 16];
#pragma unroll
    for (int gI = 0; gI < (int)(kPeerSlots / 16); ++gI) {
        cw[gI] = u4{0u, 0u, 0u, 0u};
        const int p = 16 * gI + (int)(lane / kParts);
        if (SPARSE) {
            // the peer's stream is in the sparse form: rebuild the lane's four packed words from the
            // segment of this chunk (pad words past the end of the stream have no bit set)
            if (gI < groups && p < num_peers)
                cw[gI] = sparse_words4(reinterpret_cast<const uint32_t *>(peers[p]) + (quad0 / kChunkQuads) * kSegStride,
                                       bitmaps + (16u * gI + lane / kParts) * 8u, first >> 2);
        } else if (gI < groups && p < num_peers) {
            const uint8_t *src = peers[p] + quad0 + first;
            if (!G || first + 16u <= rem_bytes) {
                typedef unsigned u4a __attribute__((ext_vector_type(4), aligned(4)));
                cw[gI] = *reinterpret_cast<const u4a *>(src);
            } else {
                // ragged end of the stream (a whole number of 32-bit words): word by word
#pragma unroll
                for (unsigned i = 0; i < 4; ++i)
                    if (first + 4u * i < rem_bytes) cw[gI][i] = *reinterpret_cast<const unsigned *>(src + 4u * i);
            }
        }
    }

    f4 g = ldgrad<G, GT>(grad, qi, cnt);
    f4 r = ld4g<G>(resid, qi, cnt);
    const f4 w = ld4g<G>(wg, qi, cnt);

    // own codes: quantise, keep the residual, write what would be pushed
    f4 sent;
    const unsigned own = quantize_quad(g, r, t, sent);
    st4g<G>(resid, qi, cnt, r);
    if (!G || qi < rem_bytes) pself[qi] = (uint8_t)own;

    // stage the peers' bytes: row p of the LDS block holds peer p's bytes of this piece
#pragma unroll
    for (int gI = 0; gI < (int)(kPeerSlots / 16); ++gI)
        if (gI < groups) *reinterpret_cast<u4 *>(lds + (16u * gI + lane / kParts) * kPieceQuads + 16u * part) = cw[gI];
    if (kPieceWaves == 1) {
        // one wave per workgroup: a wave-level release / acquire pair orders its LDS writes before its reads
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    } else {
        __syncthreads();
    }

    f4 agg = {0.0f, 0.0f, 0.0f, 0.0f};
    if (POW2) {
        // count form: four workers' bytes side by side in one register; field k of acc[c] collects
        // 2 + value for element c of the workers in byte position k
        unsigned acc[4] = {0u, 0u, 0u, 0u};
        auto add4 = [&](unsigned w4) {
            const unsigned z = ((w4 & 0x55555555u) | 0xAAAAAAAAu) - ((w4 >> 1) & 0x55555555u);
            acc[0] += z & 0x03030303u;
            acc[1] += (z >> 2) & 0x03030303u;
            acc[2] += (z >> 4) & 0x03030303u;
            acc[3] += (z >> 6) & 0x03030303u;
        };
        add4(own);  // the own byte and three empty positions
        const int words = (num_peers + 3) >> 2;
        for (int q = 0; q < words; ++q) {
            const uint8_t *row = lds + (4u * q) * kPieceQuads + lane;
            const unsigned w4 = (unsigned)row[0] | ((unsigned)row[kPieceQuads] << 8) |
                                ((unsigned)row[2 * kPieceQuads] << 16) | ((unsigned)row[3 * kPieceQuads] << 24);
            add4(w4);
        }
        // every position added 2 whether a worker stood there or not
        const float bias_t = -(2.0f * (float)(4 * words + 4)) * t;
#pragma unroll
        for (unsigned c = 0; c < 4; ++c) {
            const unsigned a = acc[c];
            const unsigned sum = (a & 0xFFu) + ((a >> 8) & 0xFFu) + ((a >> 16) & 0xFFu) + (a >> 24);
            agg[c] = __builtin_fmaf((float)sum, t, bias_t);
        }
    } else {
        // literal chain: one rounded add per worker and element, worker order, own codes at `self`
        auto chain = [&](unsigned b) {
            const unsigned sf = signed_fields(b);
#pragma unroll
            for (unsigned c = 0; c < 4; ++c) {
                const int m = ((int)(sf << (30u - 2u * c))) >> 30;
                agg[c] = __builtin_fmaf((float)m, t, agg[c]);
            }
        };
        for (int p = 0; p < self; ++p) chain(lds[(unsigned)p * kPieceQuads + lane]);
        agg = agg + sent;
        for (int p = self; p < num_peers; ++p) chain(lds[(unsigned)p * kPieceQuads + lane]);
    }

    // eq. 11 and eq. 10 from the same loaded weight
    f4 vl, vg;
#pragma unroll
    for (unsigned c = 0; c < 4; ++c) {
        vl[c] = __builtin_fmaf(-lr_local, g[c], w[c]);
        vg[c] = __builtin_fmaf(-scale, agg[c], w[c]);
    }
    if (WRITE_LOCAL) st4g<G>(wl, qi, cnt, vl);
    st4g<G>(wg, qi, cnt, vg);
    // the next piece of this workgroup overwrites the LDS block: keep its writes behind these reads
    if (kPieceWaves == 1) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    } else {
        __syncthreads();
    }
}

template <unsigned kPieceWaves, bool POW2, bool WRITE_LOCAL, int GT, bool SPARSE>
__global__ __launch_bounds__(64 * kPieceWaves) void k_fused_compressed(const TensorDesc *__restrict__ tensors,
                                                                       const ChunkRef *__restrict__ chunks,
                                                                       unsigned long long num_pieces,
                                                                       const uint8_t *const *__restrict__ peers,
                                                                       int num_peers, int self, float t_call,
                                                                       float lr_local, float scale)
{
    constexpr unsigned kPieceQuads = 64 * kPieceWaves;
    constexpr unsigned kPerChunk = kChunkQuads / kPieceQuads;
    __shared__ __attribute__((aligned(16))) uint8_t lds[kPeerSlots * kPieceQuads + (SPARSE ? kPeerSlots * 32 : 0)];
    for (unsigned long long b = blockIdx.x; b < num_pieces; b += gridDim.x) {
        const unsigned long long x = piece_of_workgroup<true>(b, kPerChunk, num_pieces);
        const ChunkRef cr = chunks[x / kPerChunk];
        const TensorDesc d = tensors[cr.tensor];
        const size_t quad0 = (size_t)cr.chunk * kChunkQuads;
        const unsigned piece = (unsigned)(x % kPerChunk);
        const uint8_t *const *tp = peers + (size_t)cr.tensor * (size_t)num_peers;
        const float t = d.threshold > 0.0f ? d.threshold : t_call;
        if (cr.chunk < d.ext.full_chunks) {
            fused_piece<kPieceWaves, false, POW2, WRITE_LOCAL, GT, SPARSE>(d, tp, num_peers, self, quad0, piece, kChunkElems,
                                                                   kChunkQuads, t, lr_local, scale, lds);
        } else if (piece * kPieceQuads < d.ext.tail_bytes) {
            // (the packed bytes of the ragged end cover its elements: pieces past them have nothing to do)
            fused_piece<kPieceWaves, true, POW2, WRITE_LOCAL, GT, SPARSE>(d, tp, num_peers, self, quad0, piece,
                                                                  d.ext.tail_elems, d.ext.tail_bytes, t, lr_local,
                                                                  scale, lds);
        }
    }
}

// Passes that use the workers' 32-bit gradients (Alg. 1: WARMUP passes and the
// correction branch of FormalTraining; eq. 1).  No quantisation, residual and
// packed streams are not touched.
//   SUM    true:  the aggregate is summed here from the N gradients, worker order,
//                 own gradient at position `self` (reads 4N + 4, writes 4 or 8 B/element)
//          false: the aggregate is read from agg_full
//   LOCAL  kLocalOnly: eq. 11 alone, w_global untouched (the local half of a split step)
//          kLocalNone: global rule only              (WARMUP, i < n-1)
//          kLocalCopy: w_local = new global weight   (WARMUP, i == n-1, the copy after the pull)
//          kLocalRule: w_local = W - lr_local * g    (WARMUP, i == n; correction passes; eq. 11)
constexpr int kLocalNone = 0, kLocalCopy = 1, kLocalRule = 2;
constexpr int kLocalOnly = 3;  // eq. 11 alone: w_local = W - lr_local * g, the global weights are left alone

// Launch shape of these passes, chosen by measurement: a workgroup is ONE wave that takes one
// quad per lane (a "piece" of 64 quads = 1 KiB of every stream; 16 pieces to a chunk), and the
// N-way sum loads the workers' gradients one after the other, each add waiting for its load.
// Memory-level parallelism comes from the number of waves (32 per compute unit), not from
// loads in flight per wave: waves that start together then walk the N streams together, so
// the requests in flight chip-wide fall on one or two streams at a time instead of all N.
// On the VGG-16-shaped list with 16 workers the sum runs at 6.2-6.3 TB/s that way; with 15
// loads in flight per wave it ran at 5.6 TB/s, and with 512-lane workgroups, two quads per lane
// and 8 loads in flight at 5.6-5.7 TB/s.
constexpr unsigned kFullBlock = CDSGD_FULL_BLOCK;            // lanes per workgroup = quads per piece
constexpr unsigned kPiecesPerChunk = kChunkQuads / kFullBlock;
static_assert(kChunkQuads % kFullBlock == 0 && kFullBlock % 64 == 0, "pieces tile a chunk, whole waves");

// One piece of one chunk: quad qi of the chunk for this lane, cnt of its elements exist.
template <bool G, bool SUM, int LOCAL, int GT>
__device__ __forceinline__ void full_piece(const TensorDesc &d, const void *const *__restrict__ pg,
                                           int num_peers, int self, size_t quad0, unsigned qi,
                                           unsigned rem_elems, float lr_local, float scale)
{
    float *__restrict__ wg = d.w_global + 4 * quad0;
    float *__restrict__ wl = d.w_local + 4 * quad0;
    const void *__restrict__ grad = grad_at<GT>(d.grad, quad0);
    const int cnt = quad_count<G>(rem_elems, qi);
    if (G && cnt == 0) return;
    const f4 w = ld4g<G>(wg, qi, cnt);
    f4 g = {0.0f, 0.0f, 0.0f, 0.0f}, a = {0.0f, 0.0f, 0.0f, 0.0f};
    if (SUM || LOCAL == kLocalRule || LOCAL == kLocalOnly) g = ldgrad<G, GT>(grad, qi, cnt);
    if (LOCAL == kLocalOnly) {
        f4 vl;
#pragma unroll
        for (unsigned c = 0; c < 4; ++c) vl[c] = __builtin_fmaf(-lr_local, g[c], w[c]);
        st4g<G>(wl, qi, cnt, vl);
        return;
    }
    if (!SUM) a = ld4g<G>(d.agg_full + 4 * quad0, qi, cnt);
    if (SUM) {
        // one gradient at a time, each add waiting for its load: see the note on the launch shape
        for (int p = 0; p < self; ++p) a = a + ldgrad<G, GT>(grad_at<GT>(pg[p], quad0), qi, cnt);
        a = a + g;
        for (int p = self; p < num_peers; ++p) a = a + ldgrad<G, GT>(grad_at<GT>(pg[p], quad0), qi, cnt);
    }
    f4 vg, vl;
#pragma unroll
    for (unsigned c = 0; c < 4; ++c) {
        vg[c] = __builtin_fmaf(-scale, a[c], w[c]);
        vl[c] = LOCAL == kLocalRule ? __builtin_fmaf(-lr_local, g[c], w[c]) : vg[c];
    }
    if (LOCAL != kLocalNone) st4g<G>(wl, qi, cnt, vl);
    st4g<G>(wg, qi, cnt, vg);
}

// peer_grads: [num_tensors][num_peers] pointers (own row left out), or unused when !SUM.
// The grid walks the pieces of the chunk table: piece x belongs to chunk slot x / kPiecesPerChunk.
template <bool SUM, int LOCAL, int GT>
__global__ __launch_bounds__(CDSGD_FULL_BLOCK) void k_fused_full(const TensorDesc *__restrict__ tensors,
                                                                 const ChunkRef *__restrict__ chunks,
                                                                 unsigned long long num_pieces,
                                                                 const void *const *__restrict__ peer_grads,
                                                                 int num_peers, int self, float lr_local,
                                                                 float scale)
{
    for (unsigned long long b = blockIdx.x; b < num_pieces; b += gridDim.x) {
        const unsigned long long x = piece_of_workgroup<CDSGD_XCD_FULL != 0>(b, kPiecesPerChunk, num_pieces);
        const ChunkRef cr = chunks[x / kPiecesPerChunk];
        const TensorDesc d = tensors[cr.tensor];
        const size_t quad0 = (size_t)cr.chunk * kChunkQuads;
        const unsigned qi = (unsigned)(x % kPiecesPerChunk) * kFullBlock + threadIdx.x;
        const void *const *pg = SUM ? peer_grads + (size_t)cr.tensor * (size_t)num_peers : nullptr;
        if (cr.chunk < d.ext.full_chunks)
            full_piece<false, SUM, LOCAL, GT>(d, pg, num_peers, self, quad0, qi, kChunkElems, lr_local, scale);
        else
            full_piece<true, SUM, LOCAL, GT>(d, pg, num_peers, self, quad0, qi, d.ext.tail_elems, lr_local, scale);
    }
}

// ---------------------------------------------------------------------------
// tables built on the device, for the entry point that allocates nothing
// ---------------------------------------------------------------------------
// Up to kStorePayload bytes travel in the kernel arguments and are written to dst.
constexpr unsigned kStorePayload = 3072;
struct StorePayload {
    uint4 q[kStorePayload / 16];
};

__global__ __launch_bounds__(256) void k_static_store(StorePayload p, uint4 *__restrict__ dst, unsigned count16)
{
    const unsigned i = threadIdx.x;
    if (i < count16) dst[i] = p.q[i];
}

// chunk_start[i] = number of chunks of tensors 0..i-1 (num_tensors + 1 entries, the last one
// the total).  Slot s of the chunk table belongs to the tensor i with
// chunk_start[i] <= s < chunk_start[i + 1].
__global__ __launch_bounds__(256) void k_static_chunks(const unsigned *__restrict__ chunk_start, int num_tensors,
                                                       ChunkRef *__restrict__ chunks, unsigned total)
{
    const unsigned slot = blockIdx.x * 256u + threadIdx.x;
    if (slot >= total) return;
    int lo = 0, hi = num_tensors;  // invariant: chunk_start[lo] <= slot < chunk_start[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (chunk_start[mid] <= slot) lo = mid;
        else hi = mid;
    }
    ChunkRef cr;
    cr.tensor = (unsigned)lo;
    cr.chunk = slot - chunk_start[lo];
    chunks[slot] = cr;
}

// Layout of the static device array: descriptor table, chunk_start, peers' pointer table,
// chunk table; every region starts on a 256-byte boundary and has room for the 16-byte
// granularity of k_static_store.
constexpr size_t round256(size_t x) { return (x + 255) & ~(size_t)255; }
constexpr int kStaticMaxTensors = CDSGD_STATIC_MAX_TENSORS;
constexpr unsigned kStaticMaxChunks = CDSGD_STATIC_MAX_CHUNKS;
constexpr size_t kStaticOffDesc = 0;
constexpr size_t kStaticOffStart = round256(sizeof(TensorDesc) * kStaticMaxTensors + 16);
constexpr size_t kStaticOffPeers = round256(kStaticOffStart + sizeof(unsigned) * (kStaticMaxTensors + 1) + 16);
constexpr size_t kStaticOffChunks =
    round256(kStaticOffPeers + sizeof(void *) * (size_t)kStaticMaxTensors * (CDSGD_MAX_WORKERS - 1) + 16);
constexpr size_t kStaticBytes = kStaticOffChunks + sizeof(ChunkRef) * (size_t)kStaticMaxChunks;
#if CDSGD_BLOCK == 512 && CDSGD_QPL == 2
static_assert(kChunkElems == CDSGD_STATIC_CHUNK_ELEMS, "the header states the chunk size the limit is counted in");
#endif

}  // namespace

// The tables of cdsgd_step_fused_static live here (about 4.6 MiB on every GPU the library
// runs on, until the process ends).  In host code this name is only a handle for
// hipGetSymbolAddress; the device address is looked up once per device (static_scratch).
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

namespace {

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
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
constexpr unsigned kQuantLanes = 64;  // lanes = quads of a piece of k_quantize_pack

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
#define CDSGD_LAUNCH_FULL_T(SUM, LOCAL, GT)                                                                    \
    hipLaunchKernelGGL((k_fused_full<SUM, LOCAL, GT>), grid, block, 0, s, plan->tensors, plan->chunks,           \
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
    hipLaunchKernelGGL(k_quantize_pack<kQuantLanes>, dim3((unsigned)units_of(n, kQuantLanes)), dim3(kQuantLanes), 0,
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
        hipLaunchKernelGGL(k_decode_sum<true>, dim3(grid), dim3(kBlock), 0, (hipStream_t)hip_stream, tab,
                           num_workers, agg, extent_of(n), threshold, bias_t);
    else
        hipLaunchKernelGGL(k_decode_sum<false>, dim3(grid), dim3(kBlock), 0, (hipStream_t)hip_stream, tab,
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
    if (n == 0 || chunks_of(n) > kMaxGrid) return CDSGD_ERR_SIZE;
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
    const unsigned grid = (unsigned)chunks_of(n);
    const Extent nn = extent_of(n);
    if (local && global)
        hipLaunchKernelGGL((k_update<true, true>), dim3(grid), dim3(kBlock), 0, s, w_global, w_local, grad_local, agg, nn, lr_local, scale);
    else if (local)
        hipLaunchKernelGGL((k_update<true, false>), dim3(grid), dim3(kBlock), 0, s, w_global, w_local, grad_local, agg, nn, lr_local, scale);
    else
        hipLaunchKernelGGL((k_update<false, true>), dim3(grid), dim3(kBlock), 0, s, w_global, w_local, grad_local, agg, nn, lr_local, scale);
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
    for (int i = 0; i < num_tensors; ++i) {
        const cdsgd_tensor &t = tensors[i];
        ht[i] = make_desc(t);
        const unsigned nc = (unsigned)chunks_of(t.n);
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
    const unsigned long long num_pieces = (unsigned long long)plan->num_chunks * (kChunkQuads / (64u * waves));
    const dim3 grid(plan->grid_size(num_pieces, 64u * waves)), block(64u * waves);
#define CDSGD_LAUNCH_COMPRESSED_S(W, POW2, LOCAL, GT, SPARSE)                                                  \
    hipLaunchKernelGGL((k_fused_compressed<W, POW2, LOCAL, GT, SPARSE>), grid, block, 0, s, plan->tensors,      \
                       plan->chunks, num_pieces, plan->peers, num_peers, plan->self, threshold, lr_local, scale)
#define CDSGD_LAUNCH_COMPRESSED_W(W, POW2, LOCAL, GT)                                                          \
    do {                                                                                                       \
        if (plan->peers_sparse) CDSGD_LAUNCH_COMPRESSED_S(W, POW2, LOCAL, GT, true);                            \
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
#undef CDSGD_LAUNCH_COMPRESSED_S
    return launch_status();
}

}  // namespace

int cdsgd_step_fused(cdsgd_plan *plan, long step, int k, float threshold, float lr_local, float lr_global,
                     void *hip_stream)
{
    return launch_formal_pass(plan, step, k, threshold, lr_local, lr_global, true, hip_stream);
}

int cdsgd_step_local(cdsgd_plan *plan, float lr_local, void *hip_stream)
{
    if (!plan) return CDSGD_ERR_NULL;
    if (!std::isfinite(lr_local)) return CDSGD_ERR_PARAM;
    const unsigned long long num_pieces = (unsigned long long)plan->num_chunks * kPiecesPerChunk;
    const dim3 grid(plan->grid_size(num_pieces, kFullBlock)), block(kFullBlock);
    hipStream_t s = (hipStream_t)hip_stream;
#define CDSGD_LAUNCH_LOCAL(GT)                                                                                 \
    hipLaunchKernelGGL((k_fused_full<false, kLocalOnly, GT>), grid, block, 0, s, plan->tensors, plan->chunks,    \
                       num_pieces, (const void *const *)nullptr, 0, plan->self, lr_local, 0.0f)
    if (plan->grad_type == kGradBF16) CDSGD_LAUNCH_LOCAL(kGradBF16);
    else if (plan->grad_type == kGradF16) CDSGD_LAUNCH_LOCAL(kGradF16);
    else CDSGD_LAUNCH_LOCAL(kGradF32);
#undef CDSGD_LAUNCH_LOCAL
    return launch_status();
}

int cdsgd_step_global(cdsgd_plan *plan, long step, int k, float threshold, float lr_global, void *hip_stream)
{
    return launch_formal_pass(plan, step, k, threshold, 0.0f, lr_global, false, hip_stream);
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
        hipLaunchKernelGGL(k_decode_sum_sparse<true>, dim3(grid), dim3(512), 0, (hipStream_t)hip_stream, tab,
                           num_workers, agg, extent_of(n), threshold, bias_t);
    else
        hipLaunchKernelGGL(k_decode_sum_sparse<false>, dim3(grid), dim3(512), 0, (hipStream_t)hip_stream, tab,
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
                        float *sink, void *hip_stream)
{
    if (num_reads < 0 || num_reads > kProbeMaxReads || num_writes < 0 || num_writes > kProbeMaxWrites ||
        num_reads + num_writes == 0)
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
#define CDSGD_PROBE(R, W) hipLaunchKernelGGL((k_probe_streams<R, W>), grid, block, 0, s, p, sink)
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
