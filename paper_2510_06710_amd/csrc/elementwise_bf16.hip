// Vectorised bf16 versions of the memory-bound glue kernels (16-byte accesses throughout).
#include "vla_internal.h"

namespace {

// Rotary on q and k plus the KV-cache write.  Input: the fp32 [M, 3H] QKV projection (rounded to bf16
// only after the rotation).  One thread per (row, head, 8-dim chunk c of the first half): it owns dims
// [8c, 8c+8) and [d/2 + 8c, d/2 + 8c + 8) of q, k and v.  q goes to its own bf16 [M, H] buffer, k to
// the [d/8][position][8] layout, v to [position][d].
__device__ __forceinline__ void load8(const float *p, float *o) {
    f32x4_t a = *(const f32x4_t *)p, b = *(const f32x4_t *)(p + 4);
#pragma unroll
    for (int e = 0; e < 4; e++) { o[e] = a[e]; o[4 + e] = b[e]; }
}
__device__ __forceinline__ bf16x8_t pack8(const float *v) {
    bf16x8_t o;
#pragma unroll
    for (int e = 0; e < 8; e++) o[e] = (bf16_t)v[e];
    return o;
}

// Sum of up to eight partial copies of two 8-float pieces (p and p + off), added in copy order; all loads are
// issued before the first addition so that their latencies overlap.
__device__ __forceinline__ void load8x2_sum(const float *p, int off, int splits, size_t split_stride, float (&a)[8], float (&b)[8]) {
    f32x4_t w[8][4];
#pragma unroll
    for (int k = 0; k < 8; k++) {
        if (k < splits) {
            const float *q = p + (size_t)k * split_stride;
            w[k][0] = *(const f32x4_t *)q; w[k][1] = *(const f32x4_t *)(q + 4);
            w[k][2] = *(const f32x4_t *)(q + off); w[k][3] = *(const f32x4_t *)(q + off + 4);
        }
    }
#pragma unroll
    for (int e = 0; e < 4; e++) { a[e] = w[0][0][e]; a[4 + e] = w[0][1][e]; b[e] = w[0][2][e]; b[4 + e] = w[0][3][e]; }
#pragma unroll
    for (int k = 1; k < 8; k++) {
        if (k < splits) {
#pragma unroll
            for (int e = 0; e < 4; e++) { a[e] += w[k][0][e]; a[4 + e] += w[k][1][e]; b[e] += w[k][2][e]; b[4 + e] += w[k][3][e]; }
        }
    }
}

__global__ void __launch_bounds__(256) rope_kv_write_bf16_kernel(bf16_t *q_out, const float *qkv, int splits, size_t split_stride,
                                                                const float2 *table,
                                                                bf16_t *kc, bf16_t *vc, size_t total, int R, int pos0,
                                                                int n_heads, int d, int pos_stride, int H) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int chunks = d >> 4, half = d >> 1;
    const int c = (int)(idx % chunks);
    const int h = (int)((idx / chunks) % n_heads);
    const size_t m = idx / ((size_t)chunks * n_heads);
    const int s = (int)(m / R), r = (int)(m % R);
    const int pos = pos0 + r;
    const float *q = qkv + m * 3 * (size_t)H + (size_t)h * d + c * 8;
    const float *k = q + H, *v = q + 2 * (size_t)H;
    float qa[8], qb[8], ka[8], kb[8], va[8], vb[8], cs[16];
    load8x2_sum(q, half, splits, split_stride, qa, qb);
    load8x2_sum(k, half, splits, split_stride, ka, kb);
    load8x2_sum(v, half, splits, split_stride, va, vb);
    const float *tb = (const float *)(table + (size_t)r * half + c * 8);     // 8 x (cos, sin)
    load8(tb, cs); load8(tb + 8, cs + 8);
    float qlo[8], qhi[8], klo[8], khi[8];
#pragma unroll
    for (int e = 0; e < 8; e++) {
        const float co = cs[2 * e], si = cs[2 * e + 1];
        qlo[e] = qa[e] * co - qb[e] * si;
        qhi[e] = qb[e] * co + qa[e] * si;
        klo[e] = ka[e] * co - kb[e] * si;
        khi[e] = kb[e] * co + ka[e] * si;
    }
    bf16_t *qo = q_out + m * (size_t)H + (size_t)h * d + c * 8;
    *(bf16x8_t *)qo = pack8(qlo);
    *(bf16x8_t *)(qo + half) = pack8(qhi);
    const size_t head = (size_t)s * n_heads + h;
    *(bf16x8_t *)(kc + ((head * (d >> 3) + c) * pos_stride + pos) * 8) = pack8(klo);
    *(bf16x8_t *)(kc + ((head * (d >> 3) + (half >> 3) + c) * pos_stride + pos) * 8) = pack8(khi);
    bf16_t *vdst = vc + (head * pos_stride + pos) * d + c * 8;
    *(bf16x8_t *)vdst = pack8(va);
    *(bf16x8_t *)(vdst + half) = pack8(vb);
}

// RMSNorm to bf16 with the row held in registers: H = 1024 * V4 floats, 256 threads, each thread owns
// V4 float4 pieces (piece j covers elements 4 * (j * 256 + t) ..): one read of x, one write of the output.
template <int V4>
__global__ void __launch_bounds__(256) rmsnorm_bf16_kernel(bf16_t *out, const float *X, const float *gain, int H,
                                                          float eps) {
    __shared__ float red[4];
    const int t = threadIdx.x;
    const f32x4_t *x = (const f32x4_t *)(X + (size_t)blockIdx.x * H);
    f32x4_t v[V4];
    float ss = 0.f;
#pragma unroll
    for (int j = 0; j < V4; j++) {
        v[j] = x[j * 256 + t];
#pragma unroll
        for (int e = 0; e < 4; e++) ss += v[j][e] * v[j][e];
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
    if ((t & 63) == 0) red[t >> 6] = ss;
    __syncthreads();
    ss = red[0] + red[1] + red[2] + red[3];
    const float r = 1.0f / sqrtf(ss / (float)H + eps);
    const f32x4_t *g = (const f32x4_t *)gain;
    bf16x4_t *o = (bf16x4_t *)(out + (size_t)blockIdx.x * H);
#pragma unroll
    for (int j = 0; j < V4; j++) {
        f32x4_t gg = g[j * 256 + t];
        bf16x4_t w;
#pragma unroll
        for (int e = 0; e < 4; e++) w[e] = (bf16_t)(v[j][e] * r * gg[e]);
        o[j * 256 + t] = w;
    }
}

// Split-K reduction of a residual projection fused with the RMSNorm that follows it: x[m] += sum of the partial
// rows (in split order, the same additions the stand-alone reduction makes), then the norm of the new row exactly
// as rmsnorm_bf16_kernel computes it.  gain == NULL: no norm output.
template <int V4>
__global__ void __launch_bounds__(256) reduce_residual_rmsnorm_kernel(bf16_t *out, float *X, const float *P, int splits,
                                                                     size_t split_stride, const float *gain, int H, float eps) {
    __shared__ float red[4];
    const int t = threadIdx.x;
    f32x4_t *x = (f32x4_t *)(X + (size_t)blockIdx.x * H);
    const f32x4_t *p0 = (const f32x4_t *)(P + (size_t)blockIdx.x * H);
    f32x4_t v[V4];
    float ss = 0.f;
    // every load of the row (partial sums and x) is issued before the first store, then the pieces are added in
    // split order
    f32x4_t w[V4][8];
#pragma unroll
    for (int j = 0; j < V4; j++) {
#pragma unroll
        for (int k = 0; k < 8; k++)
            if (k < splits) w[j][k] = *(const f32x4_t *)((const float *)(p0 + j * 256 + t) + (size_t)k * split_stride);
        v[j] = x[j * 256 + t];
    }
#pragma unroll
    for (int j = 0; j < V4; j++) {
        f32x4_t s = w[j][0];
#pragma unroll
        for (int k = 1; k < 8; k++) {
            if (k < splits) {
#pragma unroll
                for (int e = 0; e < 4; e++) s[e] += w[j][k][e];
            }
        }
        f32x4_t xv = v[j];
#pragma unroll
        for (int e = 0; e < 4; e++) xv[e] += s[e];
        x[j * 256 + t] = xv;
        v[j] = xv;
#pragma unroll
        for (int e = 0; e < 4; e++) ss += xv[e] * xv[e];
    }
    if (!gain) return;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
    if ((t & 63) == 0) red[t >> 6] = ss;
    __syncthreads();
    ss = red[0] + red[1] + red[2] + red[3];
    const float r = 1.0f / sqrtf(ss / (float)H + eps);
    const f32x4_t *g = (const f32x4_t *)gain;
    bf16x4_t *o = (bf16x4_t *)(out + (size_t)blockIdx.x * H);
#pragma unroll
    for (int j = 0; j < V4; j++) {
        f32x4_t gg = g[j * 256 + t];
        bf16x4_t w;
#pragma unroll
        for (int e = 0; e < 4; e++) w[e] = (bf16_t)(v[j][e] * r * gg[e]);
        o[j * 256 + t] = w;
    }
}

// The same norm with the output in the GEMM's k-blocked operand layout [H / 32][kb_rows][32].  A workgroup
// takes four consecutive rows, stages their bf16 results in LDS and writes each 32-column block of the four
// rows as one 256-byte run (a row on its own would leave as 64-byte pieces kb_rows * 64 bytes apart).
template <int V4>
__global__ void __launch_bounds__(256) rmsnorm_bf16_kb_kernel(bf16_t *out, const float *X, const float *gain, int M, int H,
                                                             float eps, int kb_rows) {
    __shared__ float red[4][4];
    __shared__ __attribute__((aligned(16))) bf16_t stage[4][1024 * V4];
    const int t = threadIdx.x;
    // Rows from the last one down: the GEMM before this kernel wrote the residual stream in ascending tile rows and
    // the GEMM after it starts at tile row 0, so the rows read first here and the rows that GEMM reads first are
    // the ones most recently written, part of which the memory-side cache still holds (22.1 -> 21.4 ms per 7B
    // prefill step at 256 x 288 rows).
    const int m0 = (int)(gridDim.x - 1 - blockIdx.x) * 4;
    const f32x4_t *g = (const f32x4_t *)gain;
#pragma unroll
    for (int rr = 0; rr < 4; rr++) {
        const int m = min(m0 + rr, M - 1);                 // (a clamped row is computed again and not written)
        const f32x4_t *x = (const f32x4_t *)(X + (size_t)m * H);
        f32x4_t v[V4];
        float ss = 0.f;
#pragma unroll
        for (int j = 0; j < V4; j++) {
            v[j] = x[j * 256 + t];
#pragma unroll
            for (int e = 0; e < 4; e++) ss += v[j][e] * v[j][e];
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
        if ((t & 63) == 0) red[rr][t >> 6] = ss;
        __syncthreads();
        ss = red[rr][0] + red[rr][1] + red[rr][2] + red[rr][3];
        const float r = 1.0f / sqrtf(ss / (float)H + eps);
#pragma unroll
        for (int j = 0; j < V4; j++) {
            f32x4_t gg = g[j * 256 + t];
            bf16x4_t w;
#pragma unroll
            for (int e = 0; e < 4; e++) w[e] = (bf16_t)(v[j][e] * r * gg[e]);
            *(bf16x4_t *)&stage[rr][4 * (j * 256 + t)] = w;
        }
    }
    __syncthreads();
    // 16-byte piece q: 32-column block q / 16, row (q % 16) / 4, piece q % 4 of that row's 64 bytes
    constexpr int PIECES = 4 * 1024 * V4 / 8;
    for (int q = t; q < PIECES; q += 256) {
        const int kb = q >> 4, rr = (q >> 2) & 3, pc = q & 3;
        if (m0 + rr < M)
            *(bf16x8_t *)(out + ((size_t)kb * kb_rows + m0 + rr) * 32 + pc * 8) = *(const bf16x8_t *)&stage[rr][kb * 32 + pc * 8];
    }
}

__global__ void __launch_bounds__(256) calibration_copy_kernel(f32x4_t *dst, const f32x4_t *src, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

}  // namespace

extern "C" int vla_calibration_copy(void *dst, const void *src, size_t bytes, void *stream) {
    if (!dst || !src || bytes == 0 || bytes % 16 != 0) { vla_set_error("calibration copy: NULL pointer or size not a multiple of 16"); return VLA_EINVAL; }
    calibration_copy_kernel<<<4096, 256, 0, (hipStream_t)stream>>>((f32x4_t *)dst, (const f32x4_t *)src, bytes / 16);
    return vla_check_launch("calibration_copy");
}

// Returns 1 if handled (H a multiple of 1024, at most 8192), 0 otherwise.
int try_rmsnorm_bf16(bf16_t *out, const float *X, const float *gain, int M, int H, float eps, int kb_rows, hipStream_t st) {
    if (H % 1024 != 0 || H > 8192) return 0;
    if (M == 0) return 1;
    ProfScope ps("rmsnorm", (double)M * H * 6.0, st);
    if (kb_rows) {
        const unsigned grid = (unsigned)((M + 3) / 4);
        switch (H / 1024) {
            case 1: rmsnorm_bf16_kb_kernel<1><<<grid, 256, 0, st>>>(out, X, gain, M, H, eps, kb_rows); break;
            case 2: rmsnorm_bf16_kb_kernel<2><<<grid, 256, 0, st>>>(out, X, gain, M, H, eps, kb_rows); break;
            case 3: rmsnorm_bf16_kb_kernel<3><<<grid, 256, 0, st>>>(out, X, gain, M, H, eps, kb_rows); break;
            case 4: rmsnorm_bf16_kb_kernel<4><<<grid, 256, 0, st>>>(out, X, gain, M, H, eps, kb_rows); break;
            case 5: rmsnorm_bf16_kb_kernel<5><<<grid, 256, 0, st>>>(out, X, gain, M, H, eps, kb_rows); break;
            case 6: rmsnorm_bf16_kb_kernel<6><<<grid, 256, 0, st>>>(out, X, gain, M, H, eps, kb_rows); break;
            case 7: rmsnorm_bf16_kb_kernel<7><<<grid, 256, 0, st>>>(out, X, gain, M, H, eps, kb_rows); break;
            default: rmsnorm_bf16_kb_kernel<8><<<grid, 256, 0, st>>>(out, X, gain, M, H, eps, kb_rows); break;
        }
        int rc = vla_check_launch("rmsnorm_bf16_kb");
        return rc ? rc : 1;
    }
    switch (H / 1024) {
        case 1: rmsnorm_bf16_kernel<1><<<M, 256, 0, st>>>(out, X, gain, H, eps); break;
        case 2: rmsnorm_bf16_kernel<2><<<M, 256, 0, st>>>(out, X, gain, H, eps); break;
        case 3: rmsnorm_bf16_kernel<3><<<M, 256, 0, st>>>(out, X, gain, H, eps); break;
        case 4: rmsnorm_bf16_kernel<4><<<M, 256, 0, st>>>(out, X, gain, H, eps); break;
        case 5: rmsnorm_bf16_kernel<5><<<M, 256, 0, st>>>(out, X, gain, H, eps); break;
        case 6: rmsnorm_bf16_kernel<6><<<M, 256, 0, st>>>(out, X, gain, H, eps); break;
        case 7: rmsnorm_bf16_kernel<7><<<M, 256, 0, st>>>(out, X, gain, H, eps); break;
        default: rmsnorm_bf16_kernel<8><<<M, 256, 0, st>>>(out, X, gain, H, eps); break;
    }
    int rc = vla_check_launch("rmsnorm_bf16");
    return rc ? rc : 1;
}

int try_reduce_residual_rmsnorm_bf16(bf16_t *out, float *X, const float *P, int splits, int M, int H, const float *gain,
                                     float eps, hipStream_t st) {
    if (H % 1024 != 0 || H > 8192 || splits < 1 || splits > 8) return 0;
    if (M == 0) return 1;
    ProfScope ps("reduce_residual_norm", (double)M * H * ((splits + 2) * 4.0 + (gain ? 2.0 : 0.0)), st);
    const size_t stride = (size_t)M * H;
    switch (H / 1024) {
        case 1: reduce_residual_rmsnorm_kernel<1><<<M, 256, 0, st>>>(out, X, P, splits, stride, gain, H, eps); break;
        case 2: reduce_residual_rmsnorm_kernel<2><<<M, 256, 0, st>>>(out, X, P, splits, stride, gain, H, eps); break;
        case 3: reduce_residual_rmsnorm_kernel<3><<<M, 256, 0, st>>>(out, X, P, splits, stride, gain, H, eps); break;
        case 4: reduce_residual_rmsnorm_kernel<4><<<M, 256, 0, st>>>(out, X, P, splits, stride, gain, H, eps); break;
        case 5: reduce_residual_rmsnorm_kernel<5><<<M, 256, 0, st>>>(out, X, P, splits, stride, gain, H, eps); break;
        case 6: reduce_residual_rmsnorm_kernel<6><<<M, 256, 0, st>>>(out, X, P, splits, stride, gain, H, eps); break;
        case 7: reduce_residual_rmsnorm_kernel<7><<<M, 256, 0, st>>>(out, X, P, splits, stride, gain, H, eps); break;
        default: reduce_residual_rmsnorm_kernel<8><<<M, 256, 0, st>>>(out, X, P, splits, stride, gain, H, eps); break;
    }
    int rc = vla_check_launch("reduce_residual_rmsnorm");
    return rc ? rc : 1;
}

int launch_rope_kv_write_bf16(bf16_t *q_out, const float *qkv, int splits, size_t split_stride, const float2 *table,
                              const KvView &kv, int layer, const RowsArgs &ra, int H, hipStream_t st) {
    const size_t total = (size_t)ra.n_seq * ra.R * kv.n_heads * (kv.d / 16);
    if (total == 0) return 0;
    ProfScope ps("rope_kv_write", (double)ra.n_seq * ra.R * H * (3 * 4.0 * splits + 3 * 2.0), st);
    bf16_t *kc = (bf16_t *)kv.k + (size_t)layer * kv.layer_elems;
    bf16_t *vc = (bf16_t *)kv.v + (size_t)layer * kv.layer_elems;
    rope_kv_write_bf16_kernel<<<(unsigned)((total + 255) / 256), 256, 0, st>>>(q_out, qkv, splits, split_stride, table, kc, vc, total, ra.R, ra.pos0,
                                                                              kv.n_heads, kv.d, kv.pos_stride, H);
    return vla_check_launch("rope_kv_write_bf16");
}
