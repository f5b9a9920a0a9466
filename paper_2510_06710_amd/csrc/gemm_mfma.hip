// bf16 MFMA GEMM for gfx950 (placeholder until the tiled kernel lands: declines every shape).
#include "vla_internal.h"
int try_gemm_bf16_mfma(const GemmArgs &, hipStream_t) { return 0; }
