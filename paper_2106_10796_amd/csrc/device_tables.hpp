// Device-side tables of a layer list: extents, tensor descriptors, chunk table.
#pragma once

namespace {

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

}  // namespace
