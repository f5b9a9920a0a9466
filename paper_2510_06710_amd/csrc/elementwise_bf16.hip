// Vectorised bf16 versions of the memory-bound glue kernels (16-byte accesses throughout).
#include "vla_internal.h"

namespace {

// Rotary on q and k plus the KV-cache write, bf16.  One thread per (row, head, 8-dim chunk c of the
// first half): it owns dims [8c, 8c+8) and [d/2 + 8c, d/2 + 8c + 8) of q, k and v.  q is rotated in
// place inside the QKV buffer; k goes to the [d/8][position][8] layout, v to [position][d].
__global__ void __launch_bounds__(256) rope_kv_write_bf16_kernel(bf16_t *qkv, const float2 *table, bf16_t *kc,
                                                                bf16_t *vc, size_t total, int R, int pos0,
                                                                int n_heads, int d, int pos_stride, int H) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int chunks = d >> 4, half = d >> 1;
    const int c = (int)(idx % chunks);
    const int h = (int)((idx / chunks) % n_heads);
    const size_t m = idx / ((size_t)chunks * n_heads);
    const int s = (int)(m / R), r = (int)(m % R);
    const int pos = pos0 + r;
    bf16_t *q = qkv + m * 3 * (size_t)H + (size_t)h * d + c * 8;
    bf16_t *k = q + H, *v = q + 2 * (size_t)H;
    bf16x8_t qa = *(const bf16x8_t *)q, qb = *(const bf16x8_t *)(q + half);
    bf16x8_t ka = *(const bf16x8_t *)k, kb = *(const bf16x8_t *)(k + half);
    bf16x8_t va = *(const bf16x8_t *)v, vb = *(const bf16x8_t *)(v + half);
    const f32x4_t *tb = (const f32x4_t *)(table + (size_t)r * half + c * 8);     // 8 x (cos, sin)
    bf16x8_t qlo, qhi, klo, khi;
#pragma unroll
    for (int e2 = 0; e2 < 4; e2++) {
        f32x4_t cs = tb[e2];                          // (cos, sin) of dims 2*e2 and 2*e2 + 1
#pragma unroll
        for (int u = 0; u < 2; u++) {
            const int e = 2 * e2 + u;
            const float co = cs[2 * u], si = cs[2 * u + 1];
            const float a = (float)qa[e], b = (float)qb[e], x = (float)ka[e], y = (float)kb[e];
            qlo[e] = (bf16_t)(a * co - b * si);
            qhi[e] = (bf16_t)(b * co + a * si);
            klo[e] = (bf16_t)(x * co - y * si);
            khi[e] = (bf16_t)(y * co + x * si);
        }
    }
    *(bf16x8_t *)q = qlo;
    *(bf16x8_t *)(q + half) = qhi;
    const size_t head = (size_t)s * n_heads + h;
    *(bf16x8_t *)(kc + ((head * (d >> 3) + c) * pos_stride + pos) * 8) = klo;
    *(bf16x8_t *)(kc + ((head * (d >> 3) + (half >> 3) + c) * pos_stride + pos) * 8) = khi;
    bf16_t *vdst = vc + (head * pos_stride + pos) * d + c * 8;
    *(bf16x8_t *)vdst = va;
    *(bf16x8_t *)(vdst + half) = vb;
}

}  // namespace

int launch_rope_kv_write_bf16(bf16_t *qkv, const float2 *table, const KvView &kv, int layer, const RowsArgs &ra,
                              int H, hipStream_t st) {
    const size_t total = (size_t)ra.n_seq * ra.R * kv.n_heads * (kv.d / 16);
    if (total == 0) return 0;
    ProfScope ps("rope_kv_write", (double)ra.n_seq * ra.R * H * 5 * 2.0, st);
    bf16_t *kc = (bf16_t *)kv.k + (size_t)layer * kv.layer_elems;
    bf16_t *vc = (bf16_t *)kv.v + (size_t)layer * kv.layer_elems;
    rope_kv_write_bf16_kernel<<<(unsigned)((total + 255) / 256), 256, 0, st>>>(qkv, table, kc, vc, total, ra.R, ra.pos0,
                                                                              kv.n_heads, kv.d, kv.pos_stride, H);
    return vla_check_launch("rope_kv_write_bf16");
}
