"""CD-SGD per-step data-parallel hot path on MI355X (gfx950).

The product is libcdsgd.so (HIP kernels behind the C ABI in include/cdsgd.h);
`binding` marshals torch tensors into it, `synth` makes seeded inputs and
`runner` lays a workload out in device memory and drives the calls.
"""
from . import binding  # noqa: F401
from .binding import (CdsgdError, Plan, Trainer, cdsgd_decode_sum, cdsgd_quantize_pack, cdsgd_update,  # noqa: F401
                      new_packed, packed_words)
