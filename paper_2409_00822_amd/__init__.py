"""MI355X-native row-wise top-k selection (RTop-K, arXiv 2409.00822): thin Python binding over the
C-ABI library `librtopk.so` (hand-written HIP kernels for gfx950).

The binding only marshals arguments: device pointers of torch tensors and the current HIP stream go
straight to the C entry points declared in include/rtopk.h.  There is no CPU fallback; if the
library is missing the import of `rtopk` functions fails loudly.
"""
from .rtopk import (  # noqa: F401
    RTopKError,
    lib_path,
    load_library,
    rtopk_max_m,
    rtopk_maxk_backward,
    rtopk_maxk_backward_gather,
    rtopk_maxk_dense,
    rtopk_rowwise,
    rtopk_rowwise_bf16,
    rtopk_rowwise_exact_bf16,
    rtopk_rowwise_exact_f16,
    rtopk_rowwise_f16,
    rtopk_rowwise_eps,
    rtopk_rowwise_exact,
    rtopk_rowwise_exact_smallest,
    rtopk_rowwise_smallest,
    rtopk_rowwise_exact_u8,
    rtopk_rowwise_u8,
    rtopk_status_string,
    rtopk_version,
)
