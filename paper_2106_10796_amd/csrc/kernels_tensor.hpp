// Single-tensor kernels: quantise-and-pack (a1-a3), decode-and-sum (a4), update (a5, a6).
#pragma once

namespace {

// ---------------------------------------------------------------------------
// a4: decode-and-sum (Sec. 3.2.1; sum of eq. 10)
// ---------------------------------------------------------------------------
// A lane keeps the packed bytes of its Q quads of one worker in one register: byte j = quad j.

typedef unsigned u4 __attribute__((ext_vector_type(4)));

// values of the codes of a register, as 2-bit two's-complement fields (01 -> +1, 10 -> -1, else 0)
__device__ __forceinline__ unsigned signed_fields(unsigned w)
{
    const unsigned x = w & 0x55555555u;
    const unsigned y = (w >> 1) & 0x55555555u;
    return (x ^ y) | ((y & ~x) << 1);
}

// Literal fp32 chain: agg += value(code) for the 4 Q elements of this lane (Q quads, Q <= 4),
// one rounded add per element.  The codes are first rewritten, 16 at a time,
// as 2-bit two's-complement fields so that one signed bit-field extract
// yields the multiplier.
template <unsigned Q>
__device__ __forceinline__ void chain_codes(f4 (&agg)[Q], unsigned w, float t)
{
    const unsigned s = signed_fields(w);
#pragma unroll
    for (unsigned j = 0; j < Q; ++j) {
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
template <unsigned Q>
__device__ __forceinline__ void counts_to_sum(f4 (&agg)[Q], const unsigned (&acc)[4], float t, float bias_t)
{
#pragma unroll
    for (unsigned j = 0; j < Q; ++j) {
#pragma unroll
        for (unsigned c = 0; c < 4; ++c) {
            const float cnt = (float)((acc[c] >> (8u * j)) & 0xFFu);
            agg[j][c] = __builtin_fmaf(cnt, t, bias_t);
        }
    }
}

// The workers' stream pointers of a single-tensor call; they travel in the kernel arguments.
struct StreamTable {
    const uint8_t *p[CDSGD_MAX_WORKERS];
};

// a4 for one tensor: LANES lanes per chunk (Q = 1024 / LANES quads per lane: quads tid, LANES + tid, ...),
// the workers' bytes staged through LDS.  Sixteen workers at a time, every wave fetches the chunk's 1 KiB
// of its share of them with one 128-bit load per lane and worker (a wave-uniform worker, so its pointer
// is a scalar load from the kernel arguments), the bytes go to LDS as [worker][byte], and every lane then
// reads its Q bytes of each worker back (measured on 2^27 elements, N = 16, count form, 512 lanes:
// 6.17 TB/s, against 5.6-5.8 TB/s with a byte-wide global load per worker and lane).
template <bool POW2, unsigned LANES>
__global__ __launch_bounds__(LANES) void k_decode_sum(StreamTable tab, int num_workers, float *__restrict__ agg_out,
                                                      Extent ext, float t, float bias_t)
{
    constexpr unsigned Q = kChunkQuads / LANES, kWaves = LANES / 64u;
    static_assert(kChunkQuads == 1024 && (LANES == 256 || LANES == 512), "one 128-bit load per lane covers a worker's chunk");
    __shared__ __attribute__((aligned(16))) uint8_t rows[16][kChunkQuads];
    const unsigned tid = threadIdx.x, lane = tid & 63u;
    const int wave = __builtin_amdgcn_readfirstlane((int)(tid >> 6));
    const unsigned chunk = blockIdx.x;
    const size_t quad0 = (size_t)chunk * kChunkQuads;
    const bool tail = chunk >= ext.full_chunks;
    const unsigned rem_elems = tail ? ext.tail_elems : kChunkElems;
    const unsigned rem_bytes = tail ? ext.tail_bytes : kChunkQuads;
    f4 agg[Q];
#pragma unroll
    for (unsigned j = 0; j < Q; ++j) agg[j] = f4{0.0f, 0.0f, 0.0f, 0.0f};
    unsigned acc[4] = {0u, 0u, 0u, 0u};
    for (int p0 = 0; p0 < num_workers; p0 += 16) {
        const int np = num_workers - p0 < 16 ? num_workers - p0 : 16;
        u4 cw[16 / kWaves];
#pragma unroll
        for (int h = 0; h < (int)(16 / kWaves); ++h) {
            cw[h] = u4{0u, 0u, 0u, 0u};
            const int k = wave + (int)kWaves * h;
            if (k < np) {
                const uint8_t *src = tab.p[p0 + k] + quad0 + 16u * lane;
                if (16u * lane + 16u <= rem_bytes) {
                    typedef unsigned u4a __attribute__((ext_vector_type(4), aligned(4)));
                    cw[h] = *reinterpret_cast<const u4a *>(src);
                } else {
                    // ragged end of the stream (a whole number of 32-bit words): word by word
#pragma unroll
                    for (unsigned i = 0; i < 4; ++i)
                        if (16u * lane + 4u * i < rem_bytes) cw[h][i] = *reinterpret_cast<const unsigned *>(src + 4u * i);
                }
            }
        }
#pragma unroll
        for (int h = 0; h < (int)(16 / kWaves); ++h)
            if (wave + (int)kWaves * h < np) *reinterpret_cast<u4 *>(&rows[wave + (int)kWaves * h][16u * lane]) = cw[h];
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
    float *out = agg_out + 4 * quad0;
#pragma unroll
    for (unsigned j = 0; j < Q; ++j) {
        const unsigned qi = j * LANES + tid;
        if (!tail) st4(out, qi, agg[j]);
        else st4g<true>(out, qi, quad_count<true>(rem_elems, qi), agg[j]);
    }
}

// a5 + a6 (eq. 10, eq. 11) for one tensor, both from the weight that was loaded, in single-wave pieces of
// 64 quads (`ext` in pieces, as for k_quantize_pack; measured on 2^27 elements: 6.29 TB/s against 6.02 TB/s
// for 512-lane workgroups with two quads per lane).
template <bool G, bool LOCAL, bool GLOBAL>
__device__ __forceinline__ void update_piece(float *__restrict__ wg, float *__restrict__ wl,
                                             const float *__restrict__ grad, const float *__restrict__ agg,
                                             unsigned rem_elems, float lr_local, float scale)
{
    const unsigned lane = threadIdx.x;
    const int cnt = quad_count<G>(rem_elems, lane);
    const f4 w = ld4g<G>(wg, lane, cnt);
    f4 g = {0.0f, 0.0f, 0.0f, 0.0f}, a = {0.0f, 0.0f, 0.0f, 0.0f};
    if (LOCAL) g = ld4g<G>(grad, lane, cnt);
    if (GLOBAL) a = ld4g<G>(agg, lane, cnt);
    if (LOCAL) {
        f4 v;
#pragma unroll
        for (unsigned c = 0; c < 4; ++c) v[c] = __builtin_fmaf(-lr_local, g[c], w[c]);
        st4g<G>(wl, lane, cnt, v);
    }
    if (GLOBAL) {
        f4 v;
#pragma unroll
        for (unsigned c = 0; c < 4; ++c) v[c] = __builtin_fmaf(-scale, a[c], w[c]);
        st4g<G>(wg, lane, cnt, v);
    }
}

template <bool LOCAL, bool GLOBAL>
__global__ __launch_bounds__(64) void k_update(float *__restrict__ wg, float *__restrict__ wl,
                                                     const float *__restrict__ grad, const float *__restrict__ agg,
                                                     Extent ext, float lr_local, float scale)
{
    const unsigned piece = blockIdx.x;
    const size_t quad0 = (size_t)piece * 64u;
    wg += 4 * quad0;
    if (LOCAL) {
        wl += 4 * quad0;
        grad += 4 * quad0;
    }
    if (GLOBAL) agg += 4 * quad0;
    if (piece < ext.full_chunks) update_piece<false, LOCAL, GLOBAL>(wg, wl, grad, agg, 256u, lr_local, scale);
    else update_piece<true, LOCAL, GLOBAL>(wg, wl, grad, agg, ext.tail_elems, lr_local, scale);
}

// a1-a3 for one tensor, one wave per piece of L = 64 quads (measured: 6.68 TB/s against 6.41 TB/s for
// 512-lane workgroups with two quads per lane; decode-and-sum is faster in that shape and keeps it: in
// pieces, with the workers' bytes staged through LDS as in the fused pass, it reached 4.1-5.4 TB/s against
// 5.8 TB/s, a piece of it having too little else to do).  `ext` describes the tensor in pieces: full_chunks whole pieces, then at most one
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

}  // namespace
