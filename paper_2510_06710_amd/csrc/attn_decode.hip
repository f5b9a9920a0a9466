// Single-query attention for the autoregressive decode steps (bf16 KV cache, head_dim 64 or 128).
//
// The step is pure HBM streaming: every (environment, head) pair reads its own K and V tiles once
// (multi-head attention, no query sharing).  One workgroup of four waves owns one pair (the keys are
// split over the waves so that small batches still put enough loads in flight):
//   1. scores: a lane owns one key position per 64-key chunk; K is stored [d/8][position][8], so one load
//      instruction of the wave reads 64 consecutive positions x 16 bytes = 1 KB contiguous and no
//      cross-lane reduction is needed for q.k (q is broadcast from LDS, pre-scaled by 1/sqrt(d));
//   2. softmax over all keys with two wave reductions (scores stay in registers: <= 512 keys);
//   3. P.V: V is stored [position][d]; 8 (d = 64) or 16 (d = 128) lanes cover one V row with 16-byte
//      loads, the wave covers 8 / 4 rows per instruction (1 KB contiguous), probabilities come from
//      LDS, and the row groups are summed by lane-xor steps and a four-way add through LDS.
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

// One 256-thread workgroup per (sequence, head) pair; its four waves split the keys.
template <int D>
__global__ void __launch_bounds__(256) attn_decode_kernel(bf16_t *out, const bf16_t *qbuf, const bf16_t *kc,
                                                         const bf16_t *vc, int n_heads, int nk, int pos_stride,
                                                         int H) {
    constexpr int DC = D / 8;        // 16-byte chunks per head vector
    constexpr int RPI = 64 / DC;     // V rows per wave load instruction
    constexpr int CPW = MAXCH / 4;   // key chunks of 64 per wave (chunk index = 4 * it + wave)
    __shared__ __attribute__((aligned(16))) float qs[D];
    __shared__ float ps[MAXCH * 64];
    __shared__ float red[8];
    __shared__ __attribute__((aligned(16))) float part[4][D];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int item = blockIdx.x;
    const int s = item / n_heads, h = item - s * n_heads;
    const bf16_t *q = qbuf + (size_t)s * H + (size_t)h * D;
    const float scale = 1.0f / sqrtf((float)D);
    if (threadIdx.x < D) qs[threadIdx.x] = (float)q[threadIdx.x] * scale;
    __syncthreads();

    // ---- 1. scores: wave w owns key chunks w, w + 4, ...; lane p one position of each --------------
    const bf16_t *kh = kc + (size_t)item * D * pos_stride;
    float sc[CPW];
    float mx = -INFINITY;
#pragma unroll
    for (int it = 0; it < CPW; it++) {
        sc[it] = -INFINITY;
        const int p = (it * 4 + wave) * 64 + lane;
        if (p < nk) {
            float a = 0.f;
#pragma unroll
            for (int c = 0; c < DC; c++) {
                bf16x8_t kv = *(const bf16x8_t *)(kh + ((size_t)c * pos_stride + p) * 8);
                f32x4_t q0 = *(const f32x4_t *)&qs[c * 8];
                f32x4_t q1 = *(const f32x4_t *)&qs[c * 8 + 4];
#pragma unroll
                for (int e = 0; e < 4; e++) a += q0[e] * (float)kv[e];
#pragma unroll
                for (int e = 0; e < 4; e++) a += q1[e] * (float)kv[4 + e];
            }
            sc[it] = a;
            mx = fmaxf(mx, a);
        }
    }
    // ---- 2. softmax over all keys of the workgroup ---------------------------------------------------
    mx = wave_max(mx);
    if (lane == 0) red[wave] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));     // key 0 exists, so this is finite
    float sum = 0.f;
#pragma unroll
    for (int it = 0; it < CPW; it++) {
        const float e = __expf(sc[it] - mx);                       // exp(-inf) = 0 for positions >= nk
        sc[it] = e;
        sum += e;
    }
    sum = wave_sum(sum);
    if (lane == 0) red[4 + wave] = sum;
    __syncthreads();
    const float inv = 1.0f / (red[4] + red[5] + red[6] + red[7]);
#pragma unroll
    for (int it = 0; it < CPW; it++) {
        const int p = (it * 4 + wave) * 64 + lane;
        if (p < nk) ps[p] = sc[it] * inv;
    }
    __syncthreads();

    // ---- 3. P.V: the workgroup covers 4 * RPI rows per step, wave w rows w * RPI + g ------------------
    const bf16_t *vh = vc + (size_t)item * pos_stride * D;
    const int c = lane % DC, g = lane / DC;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
    for (int pos = wave * RPI + g; pos < nk; pos += 4 * RPI) {
        bf16x8_t v = *(const bf16x8_t *)(vh + (size_t)pos * D + c * 8);
        const float pr = ps[pos];
#pragma unroll
        for (int e = 0; e < 8; e++) acc[e] += pr * (float)v[e];
    }
#pragma unroll
    for (int off = DC; off < 64; off <<= 1)
#pragma unroll
        for (int e = 0; e < 8; e++) acc[e] += __shfl_xor(acc[e], off, 64);
    if (lane < DC) {
#pragma unroll
        for (int e = 0; e < 8; e++) part[wave][c * 8 + e] = acc[e];
    }
    __syncthreads();
    if (threadIdx.x < DC) {
        bf16x8_t o;
#pragma unroll
        for (int e = 0; e < 8; e++) {
            const int i = threadIdx.x * 8 + e;
            o[e] = (bf16_t)((part[0][i] + part[1][i]) + (part[2][i] + part[3][i]));
        }
        *(bf16x8_t *)(out + (size_t)s * H + (size_t)h * D + threadIdx.x * 8) = o;
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
    if (kv.d == 128)
        attn_decode_kernel<128><<<n_items, 256, 0, st>>>(out, q, kc, vc, kv.n_heads, nk, kv.pos_stride, H);
    else
        attn_decode_kernel<64><<<n_items, 256, 0, st>>>(out, q, kc, vc, kv.n_heads, nk, kv.pos_stride, H);
    int rc = vla_check_launch("attn_decode");
    return rc ? rc : 1;
}
