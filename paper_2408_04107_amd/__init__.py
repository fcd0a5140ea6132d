"""MI355X-native latent-KV attention (FDC, arXiv 2408.04107).

The product is libfdc.so (HIP kernels for gfx950 behind a C ABI, see
include/fdc.h); this package is its thin ctypes binding. The entry points keep
their C names.
"""
from .binding import (  # noqa: F401
    FDC_APPLY, FDC_BF16, FDC_F32, FDC_FOLD, FDC_FP4, FDC_FP8, EXPORTED_SYMBOLS, FdcError, Layout, Plan, PlanParams,
    fdc_absorb_output, fdc_absorb_query, fdc_latent_attn_decode, fdc_latent_attn_decode_at, fdc_latent_attn_decode_static, fdc_latent_attn_prefill,
    fdc_plan_decode, fdc_plan_decode_device, fdc_plan_decode_paged, fdc_plan_decode_run, fdc_plan_download, fdc_plan_params_default, fdc_profile_decode_events, fdc_plan_prefill, fdc_plan_prefill_paged, fdc_plan_upload,
    fdc_project_and_absorb_query, fdc_project_latent_kv, fdc_rope_absorb_query, fdc_rope_compress_keys, fdc_select_ranks, fdc_suggest_workers, lib,
)
