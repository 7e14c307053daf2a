// bf16 MFMA flash attention for gfx950 (placeholder until the tiled kernel lands).
#include "dsk_internal.h"

hipError_t launch_attn_mfma_bf16(const AttnArgs&, hipStream_t) { return hipErrorNotSupported; }
