// bf16 MFMA GEMM for gfx950 (placeholder until the tiled kernel lands: reports "not supported",
// so the caller takes the plain-ALU kernel).
#include "dsk_internal.h"

hipError_t launch_gemm_mfma_bf16(const void*, int64_t, const void*, int64_t, void*, int64_t, const void*, int64_t, int,
                                 int, int, int, hipStream_t) {
  return hipErrorNotSupported;
}
