"""MI355X-native verification pass of TriSpec (ternary speculative decoding).

`binding` wraps the C ABI of libtrispec.so (include/trispec.h); `loader` moves caller-supplied
host arrays into device tensors; `rounds` drives draft -> proxy -> (target) rounds over the ABI;
`build` compiles the HIP sources for gfx950; `profsum` summarises rocprofv3 CSV output.
"""
from .binding import (CRIT_ENTROPY, CRIT_MARGIN, CRIT_TOP1, K_ATTN, K_GEMM, K_HEAD, TRISPEC_BF16, TRISPEC_F32,  # noqa: F401
                      KernelTimer, KVCache, Model, PagedKVCache, RESAMPLE_DIRECT, RESAMPLE_RESIDUAL, SampleDecider, TriSpecError,
                      Verifier,
                      copy_probe, lib, sample_decide)
from .loader import fill_kv_layer, model_from_arrays  # noqa: F401
from .rounds import TernaryDecoder  # noqa: F401
