// bf16 streaming decode attention for gfx950 (placeholder: declines every shape).
#include "vla_internal.h"
int try_attention_decode_bf16(bf16_t *, const bf16_t *, const KvView &, int, const RowsArgs &, int, hipStream_t) { return 0; }
