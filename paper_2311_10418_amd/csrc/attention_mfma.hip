// bf16 MFMA variable-length attention (placeholder until the kernels land: reports "unsupported"
// so that the generic kernels run).
#include "attention.hpp"

bool attn_mfma_supported(const AttnArgs&) { return false; }
ds_status attn_fwd_mfma(const AttnArgs&, hipStream_t) { return DS_EINVAL; }
ds_status attn_bwd_mfma(const AttnArgs&, hipStream_t) { return DS_EINVAL; }
