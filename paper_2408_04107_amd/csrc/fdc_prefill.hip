// Causal prefill attention on the latent cache: placeholder until the MFMA kernel lands.
#include <hip/hip_runtime.h>

#include "fdc_internal.h"

using namespace fdc;

extern "C" fdc_status fdc_latent_attn_prefill(const fdc_layout*, const fdc_plan*, const void*, const void*,
                                              const void*, float, int, void*, void*, size_t, void*) {
  FDC_FAIL(FDC_INVALID_ARG, "fdc_latent_attn_prefill: kernel not built in this library");
}
