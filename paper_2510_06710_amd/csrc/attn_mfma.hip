// bf16 MFMA prefill attention for gfx950 (placeholder: declines every shape).
#include "vla_internal.h"
size_t attention_prefill_scratch_bytes(int, int, int, int) { return 0; }
int try_attention_prefill_bf16(bf16_t *, const bf16_t *, const KvView &, int, const RowsArgs &, int, void *, hipStream_t) { return 0; }
