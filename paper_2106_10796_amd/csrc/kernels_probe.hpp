// Measurement aid: bare streaming kernel.
#pragma once

namespace {

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

}  // namespace
