"""Split-precision optimizer step for MI355X (arXiv 2309.12381): Python binding of libmpo.so.

The work is done by hand-written HIP kernels behind the C interface in
include/mpo.h; this package only marshals arguments (binding.py) and names the
synthetic workloads (synth.py).
"""
from .binding import (  # noqa: F401
    MPO_BF16, MPO_FP16, MPO_OK, MPO_ERR_ALIAS, MPO_ERR_HIP, MPO_ERR_INVALID_ARG, MPO_ERR_NOMEM,
    MPO_ERR_TOO_LARGE, MPO_ERR_UNSUPPORTED, MPO_MAX_LAYER_GRADS, MPO_NOALLOC_MAX_CHUNKS, MPO_NOALLOC_MAX_TENSORS, MPO_OPT_ADAM, MPO_OPT_SGD, MPO_ROUND_NEAREST,
    MPO_ROUND_STOCHASTIC, MPO_ROUND_TRUNC, AdamCfg, MpoError, Plan, SgdCfg, Tensor, lib,
    mpo_adam_step, mpo_adam_step_noalloc, mpo_merge, mpo_res_bytes, mpo_sgd_step, mpo_split, mpo_step_layer, tensor_array,
)
