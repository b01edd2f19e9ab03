// Kernels over a layer list: the fused compressed pass (a1-a6) and the passes on 32-bit gradients.
#pragma once

namespace {

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

// The compressed pass over the pieces a workgroup takes (the body of the two kernels below).
template <unsigned kPieceWaves, bool POW2, bool WRITE_LOCAL, int GT, bool SPARSE>
__device__ __forceinline__ void compressed_pass(const TensorDesc *__restrict__ tensors,
                                                const ChunkRef *__restrict__ chunks, unsigned long long num_pieces,
                                                const uint8_t *const *__restrict__ peers, int num_peers, int self,
                                                float t_call, float lr_local, float scale)
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

// Waves per SIMD.  With up to 16 peers the count form is left to what its registers allow (5 for packed
// peers, 6 for sparse ones: forcing 4, 6, 7 or 8 on the packed form is 0-4 % slower, forcing 5 on the
// sparse one 6 %); the literal chain has three times the arithmetic per worker and runs 3 % faster with
// the registers squeezed for 6 (4 GiB bucket: 4.70 against 4.84 ms).
template <unsigned kPieceWaves, bool POW2, bool WRITE_LOCAL, int GT, bool SPARSE>
__attribute__((amdgpu_waves_per_eu(POW2 ? 1 : 6, POW2 ? 8 : 6)))
__global__ __launch_bounds__(64 * kPieceWaves) void k_fused_compressed(const TensorDesc *__restrict__ tensors,
                                                                       const ChunkRef *__restrict__ chunks,
                                                                       unsigned long long num_pieces,
                                                                       const uint8_t *const *__restrict__ peers,
                                                                       int num_peers, int self, float t_call,
                                                                       float lr_local, float scale)
{
    compressed_pass<kPieceWaves, POW2, WRITE_LOCAL, GT, SPARSE>(tensors, chunks, num_pieces, peers, num_peers, self,
                                                                t_call, lr_local, scale);
}

// The count form for more than 16 peers: the decode's arithmetic grows with the workers, and the same
// squeeze to 6 waves per SIMD pays (VGG-16-shaped list, N = 24 / 32 / 48 / 64: 0.745 / 0.747 / 0.687 / 0.648
// of peak as the kernel above, 0.779 / 0.777 / 0.732 / 0.705 as this one).
template <bool WRITE_LOCAL, int GT, bool SPARSE>
__attribute__((amdgpu_waves_per_eu(6, 6)))
__global__ __launch_bounds__(64 * kPieceWavesMany) void k_fused_compressed_many(const TensorDesc *__restrict__ tensors,
                                                                                const ChunkRef *__restrict__ chunks,
                                                                                unsigned long long num_pieces,
                                                                                const uint8_t *const *__restrict__ peers,
                                                                                int num_peers, int self, float t_call,
                                                                                float lr_local, float scale)
{
    compressed_pass<kPieceWavesMany, true, WRITE_LOCAL, GT, SPARSE>(tensors, chunks, num_pieces, peers, num_peers, self,
                                                                    t_call, lr_local, scale);
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

}  // namespace
