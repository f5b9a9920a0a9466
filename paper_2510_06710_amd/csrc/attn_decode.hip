// Single-query attention for the autoregressive decode steps (bf16 KV cache, head_dim 64 or 128).
//
// The step is pure HBM streaming: every (environment, head) pair reads its own K and V tiles once
// (multi-head attention, no query sharing).  One wave owns one pair:
//   1. scores: lane p owns key positions p, p+64, ...; K is stored [d/8][position][8], so one load
//      instruction of the wave reads 64 consecutive positions x 16 bytes = 1 KB contiguous and no
//      cross-lane reduction is needed for q.k (q is broadcast from LDS, pre-scaled by 1/sqrt(d));
//   2. softmax over all keys with two wave reductions (scores stay in registers: <= 512 keys);
//   3. P.V: V is stored [position][d]; 8 (d = 64) or 16 (d = 128) lanes cover one V row with 16-byte
//      loads, the wave covers 8 / 4 rows per instruction (1 KB contiguous), probabilities come from
//      LDS, and the row groups are summed by two or three lane-xor steps at the end.
#include "vla_internal.h"

namespace {

constexpr int MAXCH = 8;   // key chunks of 64 held in registers => at most 512 keys

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

template <int D>
__global__ void __launch_bounds__(256) attn_decode_kernel(bf16_t *out, const bf16_t *qbuf, const bf16_t *kc,
                                                         const bf16_t *vc, int n_items, int n_heads, int nk,
                                                         int pos_stride, int H) {
    constexpr int DC = D / 8;        // 16-byte chunks per head vector
    constexpr int RPI = 64 / DC;     // V rows per wave load instruction
    __shared__ __attribute__((aligned(16))) float qs[4][D];
    __shared__ float ps[4][MAXCH * 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int item = blockIdx.x * 4 + wave;
    if (item >= n_items) return;                       // whole wave leaves; no block barrier below
    const int s = item / n_heads, h = item - s * n_heads;
    const bf16_t *q = qbuf + (size_t)s * H + (size_t)h * D;
    const float scale = 1.0f / sqrtf((float)D);
    for (int i = lane; i < D; i += 64) qs[wave][i] = (float)q[i] * scale;
    __builtin_amdgcn_wave_barrier();

    // ---- 1. scores ---------------------------------------------------------------------------
    const bf16_t *kh = kc + (size_t)item * D * pos_stride;
    const int nch = (nk + 63) >> 6;
    float sc[MAXCH];
#pragma unroll
    for (int cc = 0; cc < MAXCH; cc++) {
        sc[cc] = -INFINITY;
        if (cc < nch) {
            const int p = cc * 64 + lane;
            if (p < nk) {
                float a = 0.f;
#pragma unroll
                for (int c = 0; c < DC; c++) {
                    bf16x8_t kv = *(const bf16x8_t *)(kh + ((size_t)c * pos_stride + p) * 8);
                    f32x4_t q0 = *(const f32x4_t *)&qs[wave][c * 8];
                    f32x4_t q1 = *(const f32x4_t *)&qs[wave][c * 8 + 4];
#pragma unroll
                    for (int e = 0; e < 4; e++) a += q0[e] * (float)kv[e];
#pragma unroll
                    for (int e = 0; e < 4; e++) a += q1[e] * (float)kv[4 + e];
                }
                sc[cc] = a;
            }
        }
    }
    // ---- 2. softmax ----------------------------------------------------------------------------
    float mx = -INFINITY;
#pragma unroll
    for (int cc = 0; cc < MAXCH; cc++) mx = fmaxf(mx, sc[cc]);
    mx = wave_max(mx);
    float sum = 0.f;
#pragma unroll
    for (int cc = 0; cc < MAXCH; cc++) {
        float e = (cc < nch) ? __expf(sc[cc] - mx) : 0.f;     // exp(-inf) = 0 for masked lanes
        sc[cc] = e;
        sum += e;
    }
    sum = wave_sum(sum);
    const float inv = 1.0f / sum;
#pragma unroll
    for (int cc = 0; cc < MAXCH; cc++)
        if (cc < nch) ps[wave][cc * 64 + lane] = sc[cc] * inv;
    __builtin_amdgcn_wave_barrier();

    // ---- 3. P.V --------------------------------------------------------------------------------
    const bf16_t *vh = vc + (size_t)item * pos_stride * D;
    const int c = lane % DC, g = lane / DC;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
    for (int pos = g; pos < nk; pos += RPI) {
        bf16x8_t v = *(const bf16x8_t *)(vh + (size_t)pos * D + c * 8);
        float pr = ps[wave][pos];
#pragma unroll
        for (int e = 0; e < 8; e++) acc[e] += pr * (float)v[e];
    }
#pragma unroll
    for (int off = DC; off < 64; off <<= 1)
#pragma unroll
        for (int e = 0; e < 8; e++) acc[e] += __shfl_xor(acc[e], off, 64);
    if (lane < DC) {
        bf16x8_t o;
#pragma unroll
        for (int e = 0; e < 8; e++) o[e] = (bf16_t)acc[e];
        *(bf16x8_t *)(out + (size_t)s * H + (size_t)h * D + c * 8) = o;
    }
}

}  // namespace

int try_attention_decode_bf16(bf16_t *out, const bf16_t *q, const KvView &kv, int layer, const RowsArgs &ra,
                              int H, hipStream_t st) {
    const int nk = ra.pos0 + 1;
    if (ra.R != 1 || nk > MAXCH * 64 || (kv.d != 64 && kv.d != 128)) return 0;
    const int n_items = ra.n_seq * kv.n_heads;
    if (n_items == 0) return 1;
    const bf16_t *kc = (const bf16_t *)kv.k + (size_t)layer * kv.layer_elems;
    const bf16_t *vc = (const bf16_t *)kv.v + (size_t)layer * kv.layer_elems;
    // algorithmic bytes: K and V tiles of every (sequence, head) pair, read once
    ProfScope ps("attn_decode", 2.0 * n_items * (double)nk * kv.d * 2.0, st);
    const int grid = (n_items + 3) / 4;
    if (kv.d == 128)
        attn_decode_kernel<128><<<grid, 256, 0, st>>>(out, q, kc, vc, n_items, kv.n_heads, nk, kv.pos_stride, H);
    else
        attn_decode_kernel<64><<<grid, 256, 0, st>>>(out, q, kc, vc, n_items, kv.n_heads, nk, kv.pos_stride, H);
    int rc = vla_check_launch("attn_decode");
    return rc ? rc : 1;
}
