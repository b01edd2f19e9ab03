// Tables built on the device for the entry point that allocates nothing, and their layout.
#pragma once

namespace {

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
