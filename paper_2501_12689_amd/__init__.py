"""MI355X-native example selection for IC-Cache (stage 1 of the Example Selector).

The work is done by hand-written HIP kernels behind a C ABI (``include/iccache.h``,
built into ``libiccache.so``).  This package is the thin Python binding: it
marshals torch tensors (device memory, streams) into that ABI and nothing else.
There is no CPU or PyTorch fallback: if the library is missing, calls raise.
"""
from .binding import (  # noqa: F401
    IC_MAX_K,
    STORE_BF16,
    STORE_FP8_E4M3,
    ICError,
    Index,
    Ivf,
    ic_index_append,
    ic_index_compact,
    ic_index_create,
    ic_index_destroy,
    ic_index_invalidate,
    ic_index_scale_utility,
    ic_index_set_domains,
    ic_index_set_utility,
    ic_search,
    ic_search_domains,
    ic_search_static,
    ic_search_threshold,
    ic_self_search,
    ic_workspace_bytes,
    lib_path,
    load_library,
)
