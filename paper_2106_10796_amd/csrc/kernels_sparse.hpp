// Sparse form of a packed stream: encoder, decode-and-sum, and the word fetch the fused pass uses.
#pragma once

namespace {

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

// a4 on sparse streams, one tensor: LANES lanes per chunk as in k_decode_sum (lane tid takes quads tid,
// LANES + tid, ...), the workers' bytes staged through LDS sixteen workers at a time.  Per batch the 16 x 8
// bitmap words go to LDS first (one word per lane); then every wave rebuilds the chunk's 256 packed words
// of its share of the workers, four consecutive words per lane with one 128-bit load of the non-zero ones
// among them; then every lane picks its bytes of each worker.
template <bool POW2, unsigned LANES>
__global__ __launch_bounds__(LANES) void k_decode_sum_sparse(StreamTable tab, int num_workers,
                                                             float *__restrict__ agg_out, Extent ext, float t,
                                                             float bias_t)
{
    constexpr unsigned Q = kChunkQuads / LANES, kWaves = LANES / 64u;
    static_assert(kChunkQuads == 1024 && (LANES == 256 || LANES == 512), "four packed words per lane cover a worker's chunk");
    __shared__ __attribute__((aligned(16))) uint8_t rows[16][kChunkQuads];
    __shared__ uint32_t bitmaps[16][8];
    const unsigned tid = threadIdx.x, lane = tid & 63u;
    const int wave = __builtin_amdgcn_readfirstlane((int)(tid >> 6));
    const unsigned chunk = blockIdx.x;
    const bool tail = chunk >= ext.full_chunks;
    const unsigned rem_elems = tail ? ext.tail_elems : kChunkElems;
    f4 agg[Q];
#pragma unroll
    for (unsigned j = 0; j < Q; ++j) agg[j] = f4{0.0f, 0.0f, 0.0f, 0.0f};
    unsigned acc[4] = {0u, 0u, 0u, 0u};
    for (int p0 = 0; p0 < num_workers; p0 += 16) {
        const int np = num_workers - p0 < 16 ? num_workers - p0 : 16;
        if (tid < 128u) {
            const unsigned k = tid >> 3;
            if ((int)k < np)
                bitmaps[k][tid & 7u] =
                    (reinterpret_cast<const uint32_t *>(tab.p[p0 + (int)k]) + (size_t)chunk * kSegStride)[tid & 7u];
        }
        __syncthreads();
#pragma unroll
        for (int h = 0; h < (int)(16 / kWaves); ++h) {
            const int k = wave + (int)kWaves * h;
            if (k < np) {
                const uint32_t *seg = reinterpret_cast<const uint32_t *>(tab.p[p0 + k]) + (size_t)chunk * kSegStride;
                // (pad words past the end of the stream have no bit set: a ragged chunk needs no other care)
                *reinterpret_cast<u4 *>(&rows[k][16u * lane]) = sparse_words4(seg, bitmaps[k], 4u * lane);
            }
        }
        __syncthreads();
        for (int k = 0; k < np; ++k) {
            unsigned w = 0;
#pragma unroll
            for (unsigned j = 0; j < Q; ++j) w |= (unsigned)rows[k][j * LANES + tid] << (8u * j);
            if (POW2) count_codes(acc, w);
            else chain_codes<Q>(agg, w, t);
        }
        __syncthreads();
    }
    if (POW2) counts_to_sum<Q>(agg, acc, t, bias_t);
    float *out = agg_out + (size_t)chunk * kChunkElems;
#pragma unroll
    for (unsigned j = 0; j < Q; ++j) {
        const unsigned qi = j * LANES + tid;
        if (!tail) st4(out, qi, agg[j]);
        else st4g<true>(out, qi, quad_count<true>(rem_elems, qi), agg[j]);
    }
}

}  // namespace
