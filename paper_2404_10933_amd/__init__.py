"""MI355X-native batched evaluation of the LLMem peak-GPU-memory estimator
(arXiv 2404.10933).  The work is done by hand-written gfx950 kernels behind a C
ABI (include/llmem.h); `binding` marshals arguments to it."""
from .binding import (  # noqa: F401
    LlmemError, Tables, DeviceConfigs, load_library, library_path,
    llmem_estimate, llmem_estimate_ex, llmem_timeline_peaks, llmem_grid_generate,
    llmem_events_count, llmem_events_generate, llmem_config_bytes, llmem_events_bytes,
    llmem_strerror, llmem_abi_version, llmem_kernels_release, llmem_kernel_forms, llmem_compiled_tables, NDETAIL, DETAIL_COLUMNS,
    llmem_estimate_methods, llmem_decide, llmem_queries_generate, NDECIDE, DECISION_COLUMNS,
    llmem_sweep, llmem_sweep_reset, NSWEEP, SWEEP_GROUPS, SWEEP_COLUMNS,
)
