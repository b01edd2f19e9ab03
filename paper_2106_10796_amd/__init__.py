"""CD-SGD per-step data-parallel hot path on MI355X (gfx950).

The product is libcdsgd.so (HIP kernels behind the C ABI in include/cdsgd.h);
`binding` marshals torch tensors into it, `synth` makes seeded inputs and
`runner` lays a workload out in device memory and drives the calls.
"""
from . import binding  # noqa: F401
from .binding import (CdsgdError, Plan, StaticLayerList, Trainer, cdsgd_decode_sum,  # noqa: F401
                      cdsgd_decode_sum_sparse, cdsgd_quantize_pack, cdsgd_sparse_encode, cdsgd_step_fused_static,
                      cdsgd_update, new_packed, new_sparse, packed_words, sparse_words)
