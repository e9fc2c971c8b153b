#include "kernels.h"
namespace t5mi {
bool attn_mfma_supported(const AttnDims&) { return false; }
hipError_t launch_attn_fwd_mfma(const void*, const float*, void*, float*, const AttnDims&, hipStream_t) { return hipErrorInvalidValue; }
size_t attn_bwd_mfma_scratch_bytes(const AttnDims&) { return 0; }
hipError_t launch_attn_bwd_mfma(const void*, const void*, const void*, const float*, const float*, float*, void*, float*, void*, const AttnDims&, hipStream_t) { return hipErrorInvalidValue; }
}
