// Backward pass of the log-probability recompute: gradients of L = sum(coef * logp) with respect to the LoRA
// factors of the seven projections of every decoder layer (the policy update of appendix I-B / I-C differentiates
// the clipped surrogate through rho = exp(logp - logp_old) only; LoRA adapters: section IV-B.2).
//
// Structure.  Stored rollouts are processed in micro-batches.  For one micro-batch: (1) the forward pass of the
// recompute (its own fused kernels), keeping the residual stream at the input of every layer (fp32 [layers][rows, H]),
// and the head, which also returns logp; (2) the head's backward puts d L / d x on the rows that predict action
// tokens; (3) layers in reverse: the layer's forward is run again from its kept input, this time with unfused
// kernels that leave every intermediate the chain rule needs, then the chain rule walks back through the
// down projection, SwiGLU, gate / up, the FFN norm, the O projection, attention, the rotation, Q / K / V and the
// attention norm.  With keep_activations, (1) is instead a forward with the unfused kernels that leaves every layer's
// intermediates in a set of its own (one per layer, for one micro-batch), and (3) runs no layer a second time.  Every large contraction -- the seven forward projections and the four input-gradient products
// dY . W, which run as the same "activation x weight^T" GEMM on a transposed copy of the weights made per layer --
// goes through the library's GEMM dispatch (MFMA kernels for bf16 shapes they cover).  Attention (scores, softmax,
// its backward) runs on materialised [rows x rows] matrices per (rollout, head) with a batched tile kernel (matrix
// cores for bf16 storage, fp32 ALU for fp32 storage); the four skinny LoRA products per projection group
// (X A^T, dY B, dY^T (X A^T), (dY B)^T X) run as GEMMs on stacked, zero-padded factors.  Gradient operands of
// the GEMMs are rounded to the storage type like every other GEMM operand; all sums are fp32 and taken in a fixed
// order (no atomics), so the result is reproducible bit for bit.
#include <type_traits>
#include <vector>

#include "vla_internal.h"

namespace {

template <typename T> __device__ __forceinline__ float ld(const T *p) { return (float)*p; }
template <typename T> __device__ __forceinline__ T cvt(float v) { return (T)v; }

__device__ __forceinline__ float bsum256(float v, float *red) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}
__device__ __forceinline__ float wsum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wmax(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// ---------------------------------------------------------------------------------------------- batched tile GEMM
// C[b] (+)= alpha * op(A[b]) . op(B[b]), fp32 accumulation and output.  op(A) is m x k (A row-major [m, k], or
// [k, m] with transA), op(B) is k x n (B row-major [k, n], or [n, k] with transB).  Batch b = b1 * inner + b2 moves
// each operand by b1 * s?1 + b2 * s?2 elements.  64 x 64 output tile per 256-thread workgroup, 4 x 4 per thread, K in
// steps of 16 through LDS; every access bounds checked.  `tri`: rows and columns index the same positions and only
// keys <= query matter (causal attention): 1 = op(A)'s columns beyond the tile's last row are skipped (P . V, dS . K),
// 2 = output tiles entirely above the diagonal are skipped (scores, dP: their entries are never read).
struct BgemmArgs {
    const void *A, *B;
    float *C;
    int m, n, k, lda, ldb, ldc, transA, transB, accumulate, inner, tri;
    int c_bf16;      // matrix-core kernel only: C is bf16 (no accumulate)
    float alpha;
    long sA1, sA2, sB1, sB2, sC1, sC2;
};

template <typename TA, typename TB>
__global__ void __launch_bounds__(256) bgemm_kernel(BgemmArgs g) {
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ float As[BK][BM + 1];
    __shared__ float Bs[BK][BN + 1];
    const int b = blockIdx.z, b1 = b / g.inner, b2 = b - b1 * g.inner;
    const TA *A = (const TA *)g.A + b1 * g.sA1 + b2 * g.sA2;
    const TB *B = (const TB *)g.B + b1 * g.sB1 + b2 * g.sB2;
    float *C = g.C + b1 * g.sC1 + b2 * g.sC2;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    if (g.tri == 2 && n0 > m0 + BM - 1) return;
    const int kend = g.tri == 1 ? min(g.k, m0 + BM) : g.k;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < kend; k0 += BK) {
#pragma unroll
        for (int e = 0; e < 4; e++) {
            const int idx = e * 256 + threadIdx.x;
            {   // op(A)[m0 + i][k0 + kk]
                int i, kk;
                if (g.transA) { i = idx & 63; kk = idx >> 6; } else { kk = idx & 15; i = idx >> 4; }
                const int gi = m0 + i, gk = k0 + kk;
                float v = 0.f;
                if (gi < g.m && gk < kend) v = g.transA ? ld(A + (size_t)gk * g.lda + gi) : ld(A + (size_t)gi * g.lda + gk);
                As[kk][i] = v;
            }
            {   // op(B)[k0 + kk][n0 + j]
                int j, kk;
                if (g.transB) { kk = idx & 15; j = idx >> 4; } else { j = idx & 63; kk = idx >> 6; }
                const int gj = n0 + j, gk = k0 + kk;
                float v = 0.f;
                if (gj < g.n && gk < kend) v = g.transB ? ld(B + (size_t)gj * g.ldb + gk) : ld(B + (size_t)gk * g.ldb + gj);
                Bs[kk][j] = v;
            }
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; kk++) {
            float a[4], w[4];
#pragma unroll
            for (int i = 0; i < 4; i++) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; j++) w[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; i++)
#pragma unroll
                for (int j = 0; j < 4; j++) acc[i][j] += a[i] * w[j];
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const int gi = m0 + ty * 4 + i;
        if (gi >= g.m) continue;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const int gj = n0 + tx * 4 + j;
            if (gj >= g.n) continue;
            float *c = C + (size_t)gi * g.ldc + gj;
            const float v = g.alpha * acc[i][j];
            *c = g.accumulate ? *c + v : v;
        }
    }
}

// The same contraction on the matrix cores, for the bf16 path: 64 x 64 output tile per workgroup, four waves of
// 32 x 32 (2 x 2 blocks of v_mfma_f32_16x16x32_bf16), K in steps of 32 through LDS.  A bf16 operand is used as it is;
// an fp32 operand (probabilities, score gradients, output gradients) is split into a bf16 head and a bf16 tail and
// both enter the product (head x head, tail x head, head x tail), so the result keeps about 16 bits of either
// operand.  Sums are fp32 in a fixed order.  Same arguments, masks and bounds checks as the tile kernel above; a
// thread moves eight consecutive elements of an operand with one 16-byte load (two for fp32) where they are inside
// the matrix and 16-byte aligned, one by one otherwise.
//
// LDS tile: [64 rows][32 k] bf16 in 80-byte rows; the four 16-byte chunks of a row are permuted by (row / 8) % 4 so
// that the element-wise stores of a transposed operand (eight rows apart per lane) land in different banks.
constexpr int BG_LD = 40;
__device__ __forceinline__ int bg_col(int row, int k) { return ((((k >> 3) ^ (row >> 3)) & 3) << 3) | (k & 7); }

template <typename T> __device__ __forceinline__ void bg_load8(const T *p, float v[8]);
template <> __device__ __forceinline__ void bg_load8<float>(const float *p, float v[8]) {
    const f32x4_t a = *(const f32x4_t *)p, b = *(const f32x4_t *)(p + 4);
#pragma unroll
    for (int e = 0; e < 4; e++) { v[e] = a[e]; v[4 + e] = b[e]; }
}
template <> __device__ __forceinline__ void bg_load8<bf16_t>(const bf16_t *p, float v[8]) {
    const bf16x8_t a = *(const bf16x8_t *)p;
#pragma unroll
    for (int e = 0; e < 8; e++) v[e] = (float)a[e];
}

// Stages op(X)[row0 .. row0 + 63][k0 .. k0 + 31] into tile[0] (bf16 heads) and, for fp32 operands, tile[1] (tails).
// k_contig: X is stored [row][k] (leading dimension ldx), else [k][row].  Elements outside rows < lim, k < kend are 0.
template <typename T, bool SPLIT>
__device__ __forceinline__ void bg_stage(bf16_t (*tile)[64][BG_LD], const T *X, bool k_contig, int ldx, int row0, int lim, int k0, int kend) {
    const int t = threadIdx.x;
    float v[8];
    if (k_contig) {
        const int row = t >> 2, kk = (t & 3) * 8, gi = row0 + row, gk = k0 + kk;
        const T *p = X + (size_t)gi * ldx + gk;
        if (gi < lim && gk + 8 <= kend && ((size_t)p & 15) == 0) bg_load8<T>(p, v);
        else {
#pragma unroll
            for (int e = 0; e < 8; e++) v[e] = (gi < lim && gk + e < kend) ? ld(p + e) : 0.f;
        }
        bf16x8_t hi, lo;
#pragma unroll
        for (int e = 0; e < 8; e++) { hi[e] = (bf16_t)v[e]; lo[e] = (bf16_t)(v[e] - (float)hi[e]); }
        *(bf16x8_t *)&tile[0][row][bg_col(row, kk)] = hi;
        if constexpr (SPLIT) *(bf16x8_t *)&tile[1][row][bg_col(row, kk)] = lo;
    } else {
        const int kk = t >> 3, r0 = (t & 7) * 8, gk = k0 + kk, gi = row0 + r0;
        const T *p = X + (size_t)gk * ldx + gi;
        if (gk < kend && gi + 8 <= lim && ((size_t)p & 15) == 0) bg_load8<T>(p, v);
        else {
#pragma unroll
            for (int e = 0; e < 8; e++) v[e] = (gk < kend && gi + e < lim) ? ld(p + e) : 0.f;
        }
#pragma unroll
        for (int e = 0; e < 8; e++) {
            const bf16_t hi = (bf16_t)v[e];
            tile[0][r0 + e][bg_col(r0 + e, kk)] = hi;
            if constexpr (SPLIT) tile[1][r0 + e][bg_col(r0 + e, kk)] = (bf16_t)(v[e] - (float)hi);
        }
    }
}

template <typename TA, typename TB>
__global__ void __launch_bounds__(256) bgemm_mfma_kernel(BgemmArgs g) {
    constexpr int BM = 64, BN = 64, BK = 32;
    constexpr bool SA = sizeof(TA) == 4, SB = sizeof(TB) == 4;
    __shared__ __attribute__((aligned(16))) bf16_t As[SA ? 2 : 1][BM][BG_LD];
    __shared__ __attribute__((aligned(16))) bf16_t Bs[SB ? 2 : 1][BN][BG_LD];
    const int b = blockIdx.z, b1 = b / g.inner, b2 = b - b1 * g.inner;
    const TA *A = (const TA *)g.A + b1 * g.sA1 + b2 * g.sA2;
    const TB *B = (const TB *)g.B + b1 * g.sB1 + b2 * g.sB2;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    if (g.tri == 2 && n0 > m0 + BM - 1) return;
    const int kend = g.tri == 1 ? min(g.k, m0 + BM) : g.k;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, l16 = lane & 15, kq = lane >> 4;
    const int wm = (wave >> 1) * 32, wn = (wave & 1) * 32;
    f32x4_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
        for (int j = 0; j < 2; j++) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < kend; k0 += BK) {
        bg_stage<TA, SA>(As, A, !g.transA, g.lda, m0, g.m, k0, kend);     // op(A)[m][k]: A is [m][k] unless transposed
        bg_stage<TB, SB>(Bs, B, g.transB != 0, g.ldb, n0, g.n, k0, kend);  // op(B)[k][n]: B is [n][k] when transposed
        __syncthreads();
        bf16x8_t af[SA ? 2 : 1][2], bfr[SB ? 2 : 1][2];
#pragma unroll
        for (int p = 0; p < (SA ? 2 : 1); p++)
#pragma unroll
            for (int i = 0; i < 2; i++) { const int r = wm + 16 * i + l16; af[p][i] = *(const bf16x8_t *)&As[p][r][bg_col(r, kq * 8)]; }
#pragma unroll
        for (int p = 0; p < (SB ? 2 : 1); p++)
#pragma unroll
            for (int j = 0; j < 2; j++) { const int r = wn + 16 * j + l16; bfr[p][j] = *(const bf16x8_t *)&Bs[p][r][bg_col(r, kq * 8)]; }
        // result layout of the instruction: the lane holds the second operand's row l16 and the first operand's rows
        // 4 kq .. 4 kq + 3, so op(B) goes first and each lane ends up with four consecutive columns of one output row
#pragma unroll
        for (int i = 0; i < 2; i++)
#pragma unroll
            for (int j = 0; j < 2; j++) {
                if constexpr (SA) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfr[0][j], af[1][i], acc[i][j], 0, 0, 0);
                if constexpr (SB) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfr[1][j], af[0][i], acc[i][j], 0, 0, 0);
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfr[0][j], af[0][i], acc[i][j], 0, 0, 0);
            }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 2; i++) {
        const int gi = m0 + wm + 16 * i + l16;
        if (gi >= g.m) continue;
#pragma unroll
        for (int j = 0; j < 2; j++) {
            const int gj = n0 + wn + 16 * j + 4 * kq;
            const size_t off = (size_t)(b1 * g.sC1 + b2 * g.sC2) + (size_t)gi * g.ldc + gj;
            if (g.c_bf16) {
                bf16_t *c = (bf16_t *)g.C + off;
#pragma unroll
                for (int r = 0; r < 4; r++)
                    if (gj + r < g.n) c[r] = (bf16_t)(g.alpha * acc[i][j][r]);
                continue;
            }
            float *c = g.C + off;
            if (gj + 4 <= g.n && !g.accumulate && ((size_t)c & 15) == 0) {
                *(f32x4_t *)c = acc[i][j] * g.alpha;
                continue;
            }
#pragma unroll
            for (int r = 0; r < 4; r++) {
                if (gj + r >= g.n) continue;
                const float v = g.alpha * acc[i][j][r];
                c[r] = g.accumulate ? c[r] + v : v;
            }
        }
    }
}

// MF: the matrix-core kernel (bf16 storage); otherwise the fp32 tile kernel.
template <typename TA, typename TB, bool MF>
int bgemm(const BgemmArgs &g, int batch, hipStream_t st) {
    if (g.m <= 0 || g.n <= 0 || batch <= 0) return 0;
    ProfScope ps(MF ? "bw_attention_mfma" : "bw_attention_tiles", 2.0 * g.m * g.n * (double)g.k * batch * (g.tri ? 0.5 : 1.0), st);
    dim3 grid((g.n + 63) / 64, (g.m + 63) / 64, batch);
    if constexpr (MF) bgemm_mfma_kernel<TA, TB><<<grid, 256, 0, st>>>(g);
    else bgemm_kernel<TA, TB><<<grid, 256, 0, st>>>(g);
    return vla_check_launch("bgemm");
}

// ---------------------------------------------------------------------------------------------- elementwise pieces
__global__ void fill_kernel(float *p, size_t n, float v) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = v;
}

// rows [M, cols] fp32 -> storage type, row strides given
template <typename T>
__global__ void cast_rows_kernel(T *out, const float *in, size_t M, int cols, int ld_out, int ld_in) {
    const size_t total = M * (size_t)cols;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const size_t m = i / cols;
        const int c = (int)(i - m * cols);
        out[m * ld_out + c] = cvt<T>(in[m * ld_in + c]);
    }
}

// Rotary on the q and k thirds of the fp32 [M, 3H] projection (pairs (i, i + d/2), angle of the row's position from
// the table), v copied; everything rounded to the storage type once, after the rotation.  sign = -1 applies the
// transpose of the rotation (the backward of q and k; v passes through).
template <typename T>
__global__ void rope_rows_kernel(T *out, const float *in, const float2 *table, size_t M, int R, int H, int d, float sign) {
    const int half = d >> 1;
    const size_t per_row = (size_t)3 * (H >> 1);                 // pairs in q and k, pairs of plain elements in v
    const size_t total = M * per_row;
    for (size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (size_t)gridDim.x * 256) {
        const size_t m = idx / per_row;
        const int e = (int)(idx - m * per_row);
        const int seg = e / (H >> 1), w = e - seg * (H >> 1);   // pair w of segment seg
        const int h = w / half, i = w - h * half;
        const size_t base = m * 3 * (size_t)H + (size_t)seg * H + (size_t)h * d;
        const float a = in[base + i], b = in[base + i + half];
        if (seg == 2) { out[base + i] = cvt<T>(a); out[base + i + half] = cvt<T>(b); continue; }
        const float2 cs = table[(size_t)(m % R) * half + i];
        const float s = sign * cs.y;
        out[base + i] = cvt<T>(a * cs.x - b * s);
        out[base + i + half] = cvt<T>(b * cs.x + a * s);
    }
}

// In-place masked softmax of the score rows of one (sequence, head), rows ldp floats apart: row i sees keys 0..i, or
// all R keys from row full_from on.  One wave per row; entries outside the mask become 0.
__global__ void __launch_bounds__(256) attn_softmax_kernel(float *SP, size_t n_rows, int R, int ldp, int full_from) {
    const size_t row = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= n_rows) return;
    const int lane = threadIdx.x & 63, i = (int)(row % R);
    const int nk = i >= full_from ? R : i + 1;
    float *s = SP + row * ldp;
    float mx = -INFINITY;
    for (int j = lane; j < nk; j += 64) mx = fmaxf(mx, s[j]);
    mx = wmax(mx);
    float sum = 0.f;
    for (int j = lane; j < nk; j += 64) { const float e = expf(s[j] - mx); s[j] = e; sum += e; }
    sum = wsum(sum);
    const float inv = 1.0f / sum;
    for (int j = lane; j < R; j += 64) s[j] = j < nk ? s[j] * inv : 0.f;
}

// dS = P (dP - sum_j P dP) in place on dP; masked entries (P = 0) become 0.
__global__ void __launch_bounds__(256) attn_ds_kernel(float *dP, const float *P, size_t n_rows, int R, int ldp, int full_from) {
    const size_t row = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= n_rows) return;
    const int lane = threadIdx.x & 63, i = (int)(row % R);
    const int nk = i >= full_from ? R : i + 1;
    float *d = dP + row * ldp;
    const float *p = P + row * ldp;
    float dot = 0.f;
    for (int j = lane; j < nk; j += 64) dot += p[j] * d[j];
    dot = wsum(dot);
    for (int j = lane; j < R; j += 64) d[j] = j < nk ? p[j] * (d[j] - dot) : 0.f;
}

// act = silu(gate) * up from the fp32 [M, 2F] projection (gate columns, then up columns)
template <typename T>
__global__ void swiglu_fwd_kernel(T *act, const float *GU, size_t M, int F) {
    const size_t total = M * (size_t)F;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const size_t m = i / F;
        const int f = (int)(i - m * F);
        const float g = GU[m * 2 * F + f], u = GU[m * 2 * F + F + f];
        act[m * F + f] = cvt<T>(g / (1.0f + expf(-g)) * u);
    }
}

// d gate = d act * up * silu'(gate), d up = d act * silu(gate); silu'(t) = s (1 + t (1 - s)), s = sigmoid(t)
template <typename T>
__global__ void swiglu_bwd_kernel(T *dGU, const float *d_act, const float *GU, size_t M, int F) {
    const size_t total = M * (size_t)F;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (size_t)gridDim.x * 256) {
        const size_t m = i / F;
        const int f = (int)(i - m * F);
        const float g = GU[m * 2 * F + f], u = GU[m * 2 * F + F + f], da = d_act[i];
        const float s = 1.0f / (1.0f + expf(-g));
        dGU[m * 2 * F + f] = cvt<T>(da * u * s * (1.0f + g * (1.0f - s)));
        dGU[m * 2 * F + F + f] = cvt<T>(da * g * s);
    }
}

// dX[m] += r (g dn) - x r^3 mean(x g dn), r = (mean(x^2) + eps)^(-1/2): the backward of n = RMSNorm(x) g.  The new
// dX is also written in the storage type to dXb (the operand of the GEMMs that follow).
template <typename T>
__global__ void __launch_bounds__(256) rmsnorm_bwd_kernel(float *dX, T *dXb, const float *X, const float *gain, const float *dn, int H, float eps) {
    __shared__ float red[4];
    const float *x = X + (size_t)blockIdx.x * H, *d = dn + (size_t)blockIdx.x * H;
    float ss = 0.f, xd = 0.f;
    for (int i = threadIdx.x; i < H; i += 256) { ss += x[i] * x[i]; xd += x[i] * gain[i] * d[i]; }
    ss = bsum256(ss, red);
    xd = bsum256(xd, red);
    const float r = 1.0f / sqrtf(ss / (float)H + eps);
    const float k = r * r * r * xd / (float)H;
    float *o = dX + (size_t)blockIdx.x * H;
    T *ob = dXb + (size_t)blockIdx.x * H;
    for (int i = threadIdx.x; i < H; i += 256) {
        const float v = o[i] + (r * gain[i] * d[i] - x[i] * k);
        o[i] = v;
        ob[i] = cvt<T>(v);
    }
}

// Head forward + backward of one read-out row (one workgroup, thread k = bin k): h = RMSNorm(x) g_f, z = h . W_bins^T,
// y = z / tau, logp = y_bin - logsumexp(y); d z_k = coef / tau * ([k = bin] - p_k); d h = d z . W_bins; d x by the norm's
// backward.  Writes logp (if asked) and the row of dX (which is zero elsewhere).
template <typename T>
__global__ void __launch_bounds__(256) head_bwd_kernel(float *dX, float *logp_out, const float *X, const float *gain, const T *Wb,
                                                      const int32_t *bins, const float *coef, int A, int rows_per_seq, int row0,
                                                      int H, float eps, float inv_tau) {
    extern __shared__ float smem[];
    float *hs = smem, *dz = smem + H;          // [H], [256]
    __shared__ float red[4];
    __shared__ float stat[2];
    const int s = blockIdx.x / A, j = blockIdx.x - s * A, t = threadIdx.x;
    const size_t m = (size_t)s * rows_per_seq + row0 + j;
    const float *x = X + m * H;
    float ss = 0.f;
    for (int i = t; i < H; i += 256) ss += x[i] * x[i];
    ss = bsum256(ss, red);
    const float r = 1.0f / sqrtf(ss / (float)H + eps);
    for (int i = t; i < H; i += 256) hs[i] = x[i] * r * gain[i];
    __syncthreads();
    const T *w = Wb + (size_t)t * H;
    float z = 0.f;
    for (int i = 0; i < H; i++) z += hs[i] * ld(w + i);
    const float y = z * inv_tau;
    dz[t] = y;
    __syncthreads();
    if (t < 64) {
        float mx = fmaxf(fmaxf(dz[t], dz[t + 64]), fmaxf(dz[t + 128], dz[t + 192]));
        mx = wmax(mx);
        float sum = expf(dz[t] - mx) + expf(dz[t + 64] - mx) + expf(dz[t + 128] - mx) + expf(dz[t + 192] - mx);
        sum = wsum(sum);
        if (t == 0) { stat[0] = mx; stat[1] = logf(sum) + mx; }
    }
    __syncthreads();
    const float lse = stat[1];
    int bin = bins[(size_t)s * A + j];
    bin = min(max(bin, 0), VLA_N_BINS - 1);
    const float c = coef[(size_t)s * A + j];
    if (logp_out && t == bin) logp_out[(size_t)s * A + j] = y - lse;
    __syncthreads();
    dz[t] = c * inv_tau * ((t == bin ? 1.0f : 0.0f) - expf(y - lse));
    __syncthreads();
    // d h_i = sum_k dz_k W[k][i], then the norm's backward; a thread owns columns t, t + 256, ...
    float xd = 0.f;
    for (int i = t; i < H; i += 256) {
        float dh = 0.f;
        for (int k = 0; k < VLA_N_BINS; k++) dh += dz[k] * ld(Wb + (size_t)k * H + i);
        hs[i] = gain[i] * dh;                       // g dh (h itself is no longer needed)
        xd += x[i] * hs[i];
    }
    xd = bsum256(xd, red);
    const float k3 = r * r * r * xd / (float)H;
    float *o = dX + m * H;
    for (int i = t; i < H; i += 256) o[i] = r * hs[i] - x[i] * k3;
}

// Wt[k][col0 + n] = W[n][k]: the weight matrix [N, K] transposed into a [K, ldt] matrix at column col0 (32 x 32 tiles
// through LDS so that both sides move whole rows).
template <typename T>
__global__ void __launch_bounds__(256) transpose_kernel(T *Wt, const T *W, int N, int K, int ldt, int col0) {
    __shared__ T tile[32][33];
    const int n0 = blockIdx.y * 32, k0 = blockIdx.x * 32, tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int r = ty; r < 32; r += 8)
        if (n0 + r < N && k0 + tx < K) tile[r][tx] = W[(size_t)(n0 + r) * K + k0 + tx];
    __syncthreads();
    for (int r = ty; r < 32; r += 8)
        if (k0 + r < K && n0 + tx < N) Wt[(size_t)(k0 + r) * ldt + col0 + n0 + tx] = tile[tx][r];
}

// dst[c][r] = src[r][c] for r < rows, c < cols (src row stride ld_src, storage or fp32 source, rounded to the storage
// type), and 0 for rows <= r < ld_dst: the operand of a GEMM that contracts over the rows of src, whose K extent is
// padded to what the kernels accept.  32 x 32 tiles through LDS.
template <typename T, typename TS>
__global__ void __launch_bounds__(256) transpose_pad_kernel(T *dst, const TS *src, int rows, int cols, int ld_src, int ld_dst) {
    __shared__ float tile[32][33];
    const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32, tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int r = ty; r < 32; r += 8)
        tile[r][tx] = (r0 + r < rows && c0 + tx < cols) ? ld(src + (size_t)(r0 + r) * ld_src + c0 + tx) : 0.f;
    __syncthreads();
    for (int c = ty; c < 32; c += 8)
        if (c0 + c < cols && r0 + tx < ld_dst) dst[(size_t)(c0 + c) * ld_dst + r0 + tx] = cvt<T>(tile[tx][c]);
}

// The same for bf16 -> bf16 with 16-byte accesses on both sides: 64 x 64 tiles, a thread moves eight consecutive
// elements.  Positions r < extent of every dst row are written (zeros from `rows` on).  Needs ld_src, ld_dst and
// extent multiples of 8 and 16-byte aligned bases (the caller checks).
__global__ void __launch_bounds__(256) transpose_pad_bf16_kernel(bf16_t *dst, const bf16_t *src, int rows, int cols, int ld_src, int ld_dst, int extent) {
    __shared__ __attribute__((aligned(16))) bf16_t tile[64][72];            // 144-byte rows: 16-byte aligned, 36 banks apart
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64, t = threadIdx.x;
#pragma unroll
    for (int h = 0; h < 2; h++) {
        const int r = (t >> 3) + 32 * h, c = (t & 7) * 8;
        bf16x8_t v;
#pragma unroll
        for (int e = 0; e < 8; e++) v[e] = (bf16_t)0.f;
        if (r0 + r < rows) {
            const bf16_t *p = src + (size_t)(r0 + r) * ld_src + c0 + c;
            if (c0 + c + 8 <= cols) v = *(const bf16x8_t *)p;
            else {
#pragma unroll
                for (int e = 0; e < 8; e++) if (c0 + c + e < cols) v[e] = p[e];
            }
        }
        *(bf16x8_t *)&tile[r][c] = v;
    }
    __syncthreads();
#pragma unroll
    for (int h = 0; h < 2; h++) {
        const int c = (t >> 3) + 32 * h, r = (t & 7) * 8;
        if (c0 + c >= cols || r0 + r >= extent) continue;                   // extent is a multiple of 8: whole pieces only
        bf16x8_t v;
#pragma unroll
        for (int e = 0; e < 8; e++) v[e] = tile[r + e][c];
        *(bf16x8_t *)(dst + (size_t)(c0 + c) * ld_dst + r0 + r) = v;
    }
}

// Stacked, zero-padded LoRA factors of a group of n_p projections that share their input (q / k / v; gate / up) as
// the 256-row weight operands of two GEMMs:  Wa [256, in]: row p * rank + j = A_p[j];  Wb [256, n_p * out]: row
// p * rank + j holds B_p[:, j] in columns p * out .. (p + 1) * out and zeros elsewhere (block diagonal), so that
// X Wa^T = [X A_0^T | X A_1^T | ..] and dY Wb^T = [dY_0 B_0 | dY_1 B_1 | ..] for dY = [dY_0 | dY_1 | ..].
struct LoraGroup { const void *a[3], *b[3]; float *da[3], *db[3]; int n_p, in, out; };
template <typename T>
__global__ void pack_factors_kernel(T *Wa, T *Wb, LoraGroup g, int rank) {
    const size_t na = (size_t)256 * g.in, nb = (size_t)256 * g.n_p * g.out;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < na + nb; i += (size_t)gridDim.x * 256) {
        if (i < na) {
            const int row = (int)(i / g.in), c = (int)(i - (size_t)row * g.in), p = row / rank, j = row - p * rank;
            Wa[i] = p < g.n_p ? ((const T *)g.a[p])[(size_t)j * g.in + c] : cvt<T>(0.f);
        } else {
            const size_t k = i - na;
            const int w = g.n_p * g.out, row = (int)(k / w), c = (int)(k - (size_t)row * w), p = row / rank, j = row - p * rank;
            const bool in_block = p < g.n_p && c >= p * g.out && c < (p + 1) * g.out;
            Wb[k] = in_block ? ((const T *)g.b[p])[(size_t)(c - p * g.out) * rank + j] : cvt<T>(0.f);
        }
    }
}

// dB_p[o][j] (+)= scale * Cb[p * out + o][p * rank + j];  dA_p[j][i] (+)= scale * Ca[i][p * rank + j]
__global__ void unpack_grads_kernel(LoraGroup g, const float *Cb, const float *Ca, int rank, float scale, int accumulate) {
    const size_t nb = (size_t)g.n_p * g.out * rank, na = (size_t)g.n_p * rank * g.in;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nb + na; i += (size_t)gridDim.x * 256) {
        if (i < nb) {
            const int p = (int)(i / ((size_t)g.out * rank));
            const size_t k = i - (size_t)p * g.out * rank;
            const int o = (int)(k / rank), j = (int)(k - (size_t)o * rank);
            const float v = scale * Cb[((size_t)p * g.out + o) * 256 + p * rank + j];
            g.db[p][k] = accumulate ? g.db[p][k] + v : v;
        } else {
            const size_t q = i - nb;
            const int p = (int)(q / ((size_t)rank * g.in));
            const size_t k = q - (size_t)p * rank * g.in;
            const int j = (int)(k / g.in), c = (int)(k - (size_t)j * g.in);
            const float v = scale * Ca[(size_t)c * 256 + p * rank + j];
            g.da[p][k] = accumulate ? g.da[p][k] + v : v;
        }
    }
}

inline unsigned blocks_for(size_t n) { size_t b = (n + 255) / 256; return (unsigned)(b > 65535 * 16 ? 65535 * 16 : (b ? b : 1)); }

// ---------------------------------------------------------------------------------------------- workspace
// What the backward of one layer reads of that layer's forward: its input and the stream after the attention block
// (fp32 [M, H]), the norm outputs, the rotated q | k | v rows, the attention probabilities
// ([rollouts * heads][rows, rows padded to 4] fp32), the attention output, the gate | up pre-activations (fp32) and the
// SwiGLU output.
struct Acts {
    float *x_in, *x_mid, *GU, *SP;
    void *Nrm, *QKVr, *AO, *Nrm2, *ACT;
};

struct BwSpace {
    float *X, *dX, *ckpt, *QKV, *Tmp, *dP, *UV, *Cab;
    void *dGU, *dXb, *dQKVb, *Wt, *Wa, *Wb, *UVt, *Xt, *dYt;
    // keep = false: one Acts set, refilled per layer by running the layer again from ckpt[l] (the first pass is the
    // recompute's fused forward, its scratch is fw).  keep = true: one set per layer, filled by the first pass.
    bool keep;
    Acts one;
    char *acts_base;
    size_t acts_stride;
    void *fw;        // scratch of the first forward pass (vla_forward_streams)
    void *split;     // partial products of the split-K LoRA GEMMs
    size_t split_bytes;
    int kp;          // rows of a micro-batch rounded up to what a GEMM's K extent accepts
    float2 *rope;
    int a_rows;
    size_t total;
};

size_t al(size_t v) { return (v + 255) & ~(size_t)255; }

// One Acts set laid out from `base` (NULL: only sized); with_streams: the set owns x_in and x_mid.
Acts plan_acts(const vla_config &c, char *base, size_t M, size_t Mp, int mb, int R, bool with_streams, size_t *bytes) {
    Acts a{};
    size_t off = 0;
    const size_t es = c.dtype == VLA_DTYPE_F32 ? 4 : 2, H = c.hidden, F = c.ffn, Rp = ((size_t)R + 3) & ~(size_t)3;
    auto take = [&](size_t b) { char *p = base ? base + off : nullptr; off += al(b); return (void *)p; };
    if (with_streams) { a.x_in = (float *)take(M * H * 4); a.x_mid = (float *)take(M * H * 4); }
    a.GU = (float *)take(M * 2 * F * 4);
    a.SP = (float *)take((size_t)mb * c.n_heads * R * Rp * 4);     // score rows start 16-byte aligned
    a.Nrm = take(Mp * H * es);
    a.QKVr = take(Mp * 3 * H * es);
    a.AO = take(Mp * H * es);
    a.Nrm2 = take(Mp * H * es);
    a.ACT = take(Mp * F * es);
    *bytes = off;
    return a;
}

BwSpace plan_bw(const vla_config &c, char *base, int mb, int R, int /*rank*/, bool keep) {
    BwSpace w;
    size_t off = 0;
    const size_t es = c.dtype == VLA_DTYPE_F32 ? 4 : 2, M = (size_t)mb * R, H = c.hidden, F = c.ffn, L = c.n_layers;
    const size_t Mp = (M + 255) / 256 * 256 + VLA_KB_PAD_ROWS;
    const size_t Rp = ((size_t)R + 3) & ~(size_t)3;
    auto take = [&](size_t bytes) { char *p = base ? base + off : nullptr; off += al(bytes); return (void *)p; };
    w.a_rows = (int)Mp;
    w.keep = keep;
    w.X = (float *)take(M * H * 4);
    w.dX = (float *)take(M * H * 4);
    w.QKV = (float *)take(M * 3 * H * 4);
    w.Tmp = (float *)take(M * (F > 3 * H ? F : 3 * H) * 4);
    w.dP = (float *)take((size_t)mb * c.n_heads * R * Rp * 4);
    // LoRA products (see lora_group): U | V [2][M, 256] fp32, their rounded transposes [2][256 + pad, kp], the stacked
    // factors, the transposed activations / output gradients and the two [dim, 256] results
    const size_t kp = M < 256 ? 256 : (M + 63) / 64 * 64, wide = 3 * H > 2 * F ? 3 * H : 2 * F, dim_p = (wide + 255) / 256 * 256 + VLA_KB_PAD_ROWS;
    w.kp = (int)kp;
    w.UV = (float *)take(2 * M * 256 * 4);
    w.Cab = (float *)take(2 * dim_p * 256 * 4);
    w.Wa = take((size_t)(256 + VLA_KB_PAD_ROWS) * (H > F ? H : F) * es);
    w.Wb = take((size_t)(256 + VLA_KB_PAD_ROWS) * wide * es);
    w.UVt = take(2 * (size_t)(256 + VLA_KB_PAD_ROWS) * kp * es);
    w.Xt = take(dim_p * kp * es);
    w.dYt = take(dim_p * kp * es);
    w.dGU = take(Mp * 2 * F * es);
    w.dXb = take(Mp * H * es);
    w.dQKVb = take(Mp * 3 * H * es);
    w.Wt = take((3 * H > 2 * F ? 3 * H : 2 * F) * H * es);      // the widest transposed stack: [H, 3H] or [H, 2F] ([F, H] is smaller)
    w.rope = (float2 *)take((size_t)R * (H / c.n_heads / 2) * sizeof(float2));
    w.split_bytes = (size_t)8 * (M > dim_p ? M : dim_p) * 256 * 4;      // up to 8 parts of the tallest [rows, 256] product
    w.split = take(w.split_bytes);
    size_t set_bytes = 0;
    if (keep) {
        plan_acts(c, nullptr, M, Mp, mb, R, true, &set_bytes);
        w.acts_stride = set_bytes;
        w.acts_base = (char *)take(set_bytes * L);
        w.one = Acts{};
        w.ckpt = nullptr;
        w.fw = nullptr;
    } else {
        plan_acts(c, nullptr, M, Mp, mb, R, false, &set_bytes);
        char *b = (char *)take(set_bytes);
        w.one = plan_acts(c, b, M, Mp, mb, R, false, &set_bytes);
        w.acts_base = nullptr;
        w.acts_stride = 0;
        w.ckpt = (float *)take(L * M * H * 4);
        w.fw = take(vla_forward_streams_bytes(c, mb, R));
    }
    w.total = off;
    return w;
}

int bw_micro_batch(const vla_config &c, int N) { return N < c.max_batch ? N : c.max_batch; }

// ---------------------------------------------------------------------------------------------- the pass itself
template <typename T>
struct Backward {
    const vla_model *m;
    const vla_config &c;
    BwSpace ws;
    hipStream_t st;
    int n, R, M, H, F, d, nh, full_from, rank;
    float scale;
    int ws_mb;       // rollouts per micro-batch the workspace is laid out for
    static constexpr bool MF = sizeof(T) == 2;      // bf16 storage: attention matrices on the matrix cores

    int gemm(const void *A, const void *W0, const void *W1, const void *W2, int n_seg, int segN, float *C, int K, int epilogue = EPI_STORE) {
        GemmArgs g{};
        g.A = A; g.W[0] = W0; g.W[1] = W1; g.W[2] = W2; g.n_seg = n_seg; g.segN = segN; g.C = C; g.M = M; g.K = K;
        g.epilogue = epilogue; g.a_rows = ws.a_rows;
        return vla_gemm_dispatch(c, g, st);
    }
    int transpose(const void *W, int N, int K, int ldt, int col0) {
        if constexpr (std::is_same_v<T, bf16_t>) {
            if (N % 8 == 0 && K % 8 == 0 && ldt % 8 == 0 && col0 % 8 == 0 && ((size_t)W & 15) == 0) {
                dim3 grid((K + 63) / 64, (N + 63) / 64);
                transpose_pad_bf16_kernel<<<grid, 256, 0, st>>>((bf16_t *)ws.Wt + col0, (const bf16_t *)W, N, K, K, ldt, N);
                return vla_check_launch("transpose");
            }
        }
        dim3 grid((K + 31) / 32, (N + 31) / 32);
        transpose_kernel<T><<<grid, 256, 0, st>>>((T *)ws.Wt, (const T *)W, N, K, ldt, col0);
        return vla_check_launch("transpose");
    }
    int cast(void *out, const float *in, int cols, int ld_out, int ld_in) {
        cast_rows_kernel<T><<<blocks_for((size_t)M * cols), 256, 0, st>>>((T *)out, in, (size_t)M, cols, ld_out, ld_in);
        return vla_check_launch("cast_rows");
    }
    BgemmArgs heads(const void *A, int lda, long sA1, long sA2, const void *B, int ldb, long sB1, long sB2, float *C, int ldc,
                    long sC1, long sC2, int mm, int nn, int kk, int tA, int tB, float alpha, int tri) {
        BgemmArgs g{};
        g.A = A; g.B = B; g.C = C; g.m = mm; g.n = nn; g.k = kk; g.lda = lda; g.ldb = ldb; g.ldc = ldc; g.transA = tA; g.transB = tB;
        g.accumulate = 0; g.inner = nh; g.tri = tri; g.alpha = alpha;
        g.sA1 = sA1; g.sA2 = sA2; g.sB1 = sB1; g.sB2 = sB2; g.sC1 = sC1; g.sC2 = sC2;
        return g;
    }

    // The activation set of layer l: its own (keep) or the shared one, whose streams are ckpt[l] and ws.X.
    Acts acts(int l) const {
        if (ws.keep) {
            size_t bytes;
            return plan_acts(c, ws.acts_base + (size_t)l * ws.acts_stride, (size_t)ws_mb * R, (size_t)ws.a_rows, ws_mb, R, true, &bytes);
        }
        Acts a = ws.one;
        a.x_in = ws.ckpt + (size_t)l * M * H;        // (the first pass packs the streams of the current micro-batch)
        a.x_mid = ws.X;
        return a;
    }
    int copy_stream(float *dst, const float *src) {
        if (dst == src) return 0;
        if (hipMemcpyAsync(dst, src, (size_t)M * H * 4, hipMemcpyDeviceToDevice, st) != hipSuccess) { vla_set_error("backward: copy failed"); return VLA_EHIP; }
        return 0;
    }

    // Layer l forward on the stream in ws.X with unfused kernels that leave in `a` everything its backward reads.
    // with_down = false stops at the SwiGLU output (a layer run again for its backward: nothing reads its output) and
    // leaves ws.X = the stream after the attention block.
    int layer_forward(int l, const Acts &a, bool with_down) {
        const vla_layer_weights &lw = m->layers[l];
        const T *Q = (const T *)a.QKVr;
        const int Rp = (R + 3) & ~3;
        const long RR = (long)R * Rp, rowsH3 = (long)R * 3 * H;
        const bool causal = full_from >= R;
        int rc;
        if (ws.keep && (rc = copy_stream(a.x_in, ws.X))) return rc;          // (otherwise ws.X was loaded from there)
        if ((rc = launch_rmsnorm<T>((T *)a.Nrm, ws.X, (const float *)lw.attn_norm, M, H, c.rms_eps, st))) return rc;
        if ((rc = gemm(a.Nrm, lw.wq, lw.wk, lw.wv, 3, H, ws.QKV, H))) return rc;
        rope_rows_kernel<T><<<blocks_for((size_t)M * 3 * (H / 2)), 256, 0, st>>>((T *)a.QKVr, ws.QKV, ws.rope, (size_t)M, R, H, d, 1.0f);
        if ((rc = vla_check_launch("rope_rows"))) return rc;
        // scores = q k^T / sqrt(d) per (sequence, head); softmax under the mask; output = P v
        BgemmArgs g = heads(Q, 3 * H, rowsH3, d, Q + H, 3 * H, rowsH3, d, a.SP, Rp, RR * nh, RR, R, R, d, 0, 1, 1.0f / sqrtf((float)d), causal ? 2 : 0);
        if ((rc = bgemm<T, T, MF>(g, n * nh, st))) return rc;
        attn_softmax_kernel<<<(unsigned)(((size_t)n * nh * R + 3) / 4), 256, 0, st>>>(a.SP, (size_t)n * nh * R, R, Rp, full_from);
        if ((rc = vla_check_launch("attn_softmax"))) return rc;
        g = heads(a.SP, Rp, RR * nh, RR, Q + 2 * H, 3 * H, rowsH3, d, MF ? (float *)a.AO : ws.Tmp, H, (long)R * H, d, R, d, R, 0, 0, 1.0f, causal ? 1 : 0);
        g.c_bf16 = MF;                               // the matrix-core kernel rounds the output to the storage type itself
        if ((rc = bgemm<float, T, MF>(g, n * nh, st))) return rc;
        if (!MF && (rc = cast(a.AO, ws.Tmp, H, H, H))) return rc;
        if ((rc = gemm(a.AO, lw.wo, nullptr, nullptr, 1, H, ws.X, H, EPI_RESIDUAL))) return rc;     // x_mid = x_in + O(...)
        if ((rc = copy_stream(a.x_mid, ws.X))) return rc;
        if ((rc = launch_rmsnorm<T>((T *)a.Nrm2, ws.X, (const float *)lw.ffn_norm, M, H, c.rms_eps, st))) return rc;
        if ((rc = gemm(a.Nrm2, lw.w_gate, lw.w_up, nullptr, 2, F, a.GU, H))) return rc;
        swiglu_fwd_kernel<T><<<blocks_for((size_t)M * F), 256, 0, st>>>((T *)a.ACT, a.GU, (size_t)M, F);
        if ((rc = vla_check_launch("swiglu_fwd"))) return rc;
        if (!with_down) return 0;
        return gemm(a.ACT, lw.w_down, nullptr, nullptr, 1, H, ws.X, F, EPI_RESIDUAL);
    }

    // LoRA gradients of a group of projections that share their input X [M, in] (storage type, contiguous rows) and
    // whose output gradients sit side by side in dY [M, n_p * out]: four GEMMs on the MFMA path where the shape allows,
    //   U = X Wa^T, V = dY Wb^T                                   [M, 256]   (Wa, Wb: the stacked, zero-padded factors)
    //   Cb = dY^T U = (dY^T)[n_p * out, kp] . (U^T)[256, kp]^T    -> dB_p = scale * its block p
    //   Ca = X^T V  = (X^T)[in, kp] . (V^T)[256, kp]^T            -> dA_p = scale * its block p, transposed
    // with U, V rounded to the storage type like every GEMM operand and the contraction over the rows padded with zeros
    // to kp.  Needs n_p * rank <= 256.
    int gemm_rows(const void *A, const void *W, float *C, int rows, int a_rows, int K) {
        GemmArgs g{};
        g.A = A; g.W[0] = W; g.n_seg = 1; g.segN = 256; g.C = C; g.M = rows; g.K = K; g.epilogue = EPI_STORE; g.a_rows = a_rows;
        g.split_scratch = ws.split; g.split_scratch_bytes = ws.split_bytes;     // few output tiles: cut K into parts
        return vla_gemm_dispatch(c, g, st);
    }
    int lora_group(LoraGroup lg, const void *X, const void *dY, bool first) {
        const int in = lg.in, wout = lg.n_p * lg.out, kp = ws.kp;
        const int pad_rows = 256 + VLA_KB_PAD_ROWS;
        float *U = ws.UV, *V = ws.UV + (size_t)M * 256, *Cb = ws.Cab, *Ca = ws.Cab + (size_t)((wout + 255) / 256 * 256 + VLA_KB_PAD_ROWS) * 256;
        T *Ut = (T *)ws.UVt, *Vt = Ut + (size_t)pad_rows * kp;
        int rc;
        pack_factors_kernel<T><<<blocks_for((size_t)256 * (in + wout)), 256, 0, st>>>((T *)ws.Wa, (T *)ws.Wb, lg, rank);
        if ((rc = vla_check_launch("pack_factors"))) return rc;
        if ((rc = gemm_rows(X, ws.Wa, U, M, ws.a_rows, in)) || (rc = gemm_rows(dY, ws.Wb, V, M, ws.a_rows, wout))) return rc;
        auto tp = [&](auto *dst, auto *src, int rows, int cols, int ld_src) {
            ProfScope ps("bw_transpose", 0.0, st);
            using D = std::remove_pointer_t<decltype(dst)>;
            using S = std::remove_const_t<std::remove_pointer_t<decltype(src)>>;
            if constexpr (std::is_same_v<D, bf16_t> && std::is_same_v<S, bf16_t>) {
                if (ld_src % 8 == 0 && kp % 8 == 0 && ((size_t)dst & 15) == 0 && ((size_t)src & 15) == 0) {
                    dim3 grid((cols + 63) / 64, (kp + 63) / 64);
                    transpose_pad_bf16_kernel<<<grid, 256, 0, st>>>(dst, src, rows, cols, ld_src, kp, kp);
                    return vla_check_launch("transpose_pad");
                }
            }
            dim3 grid((cols + 31) / 32, (kp + 31) / 32);
            transpose_pad_kernel<<<grid, 256, 0, st>>>(dst, src, rows, cols, ld_src, kp);
            return vla_check_launch("transpose_pad");
        };
        if ((rc = tp(Ut, (const float *)U, M, 256, 256)) || (rc = tp(Vt, (const float *)V, M, 256, 256))) return rc;
        if ((rc = tp((T *)ws.Xt, (const T *)X, M, in, in)) || (rc = tp((T *)ws.dYt, (const T *)dY, M, wout, wout))) return rc;
        const int rows_b = (wout + 255) / 256 * 256 + VLA_KB_PAD_ROWS, rows_a = (in + 255) / 256 * 256 + VLA_KB_PAD_ROWS;
        if ((rc = gemm_rows(ws.dYt, Ut, Cb, wout, rows_b, kp)) || (rc = gemm_rows(ws.Xt, Vt, Ca, in, rows_a, kp))) return rc;
        unpack_grads_kernel<<<blocks_for((size_t)lg.n_p * rank * (lg.out + in)), 256, 0, st>>>(lg, Cb, Ca, rank, scale, first ? 0 : 1);
        return vla_check_launch("unpack_grads");
    }
    static LoraGroup group_of(int n_p, const vla_lora_factor *f, const vla_lora_grad *g, int in, int out) {
        LoraGroup lg{};
        lg.n_p = n_p; lg.in = in; lg.out = out;
        for (int p = 0; p < n_p; p++) { lg.a[p] = f[p].a; lg.b[p] = f[p].b; lg.da[p] = g[p].da; lg.db[p] = g[p].db; }
        return lg;
    }

    // Backward of layer l: on entry ws.dX (and ws.dXb, its copy in the storage type) = d L / d x_out; on exit
    // d L / d x_in.
    int layer_backward(int l, const vla_lora_layer &lo, const vla_lora_layer_grads &gr, bool first) {
        const vla_layer_weights &lw = m->layers[l];
        const Acts a = acts(l);
        const T *Q = (const T *)a.QKVr;
        const int Rp = (R + 3) & ~3;
        const long RR = (long)R * Rp, rowsH3 = (long)R * 3 * H;
        const bool causal = full_from >= R;
        const float isd = 1.0f / sqrtf((float)d);
        int rc;
        if (!ws.keep) {                              // run the layer again from its kept input
            if ((rc = copy_stream(ws.X, a.x_in))) return rc;
            if ((rc = layer_forward(l, a, false))) return rc;
        }
        // ---- down projection and SwiGLU (ws.dXb: ws.dX in the storage type, left by the head or the layer above)
        if ((rc = lora_group(group_of(1, &lo.down, &gr.down, F, H), a.ACT, ws.dXb, first))) return rc;
        if ((rc = transpose(lw.w_down, H, F, H, 0))) return rc;                               // [F, H]
        if ((rc = gemm(ws.dXb, ws.Wt, nullptr, nullptr, 1, F, ws.Tmp, H))) return rc;          // d act [M, F]
        swiglu_bwd_kernel<T><<<blocks_for((size_t)M * F), 256, 0, st>>>((T *)ws.dGU, ws.Tmp, a.GU, (size_t)M, F);
        if ((rc = vla_check_launch("swiglu_bwd"))) return rc;
        if ((rc = lora_group(group_of(2, &lo.gate, &gr.gate, H, F), a.Nrm2, ws.dGU, first))) return rc;   // gate, up adjacent in the structs
        if ((rc = transpose(lw.w_gate, F, H, 2 * F, 0)) || (rc = transpose(lw.w_up, F, H, 2 * F, F))) return rc;   // [H, 2F]
        if ((rc = gemm(ws.dGU, ws.Wt, nullptr, nullptr, 1, H, ws.Tmp, 2 * F))) return rc;      // d n2 [M, H]
        rmsnorm_bwd_kernel<T><<<M, 256, 0, st>>>(ws.dX, (T *)ws.dXb, a.x_mid, (const float *)lw.ffn_norm, ws.Tmp, H, c.rms_eps);
        if ((rc = vla_check_launch("rmsnorm_bwd"))) return rc;
        // ---- O projection and attention (ws.dX, ws.dXb are now d L / d x_mid)
        if ((rc = lora_group(group_of(1, &lo.o, &gr.o, H, H), a.AO, ws.dXb, first))) return rc;
        if ((rc = transpose(lw.wo, H, H, H, 0))) return rc;
        float *d_ao = a.GU;                          // [M, H] fp32; the gate / up pre-activations are no longer needed
        if ((rc = gemm(ws.dXb, ws.Wt, nullptr, nullptr, 1, H, d_ao, H))) return rc;
        float *dqkv = ws.Tmp;                        // [M, 3H] fp32: d q | d k | d v (q, k still in the rotated frame)
        // dP = dO v^T ; dV = P^T dO ; dS = P (dP - rowsum(P dP)) ; dQ = dS k / sqrt(d) ; dK = dS^T q / sqrt(d)
        BgemmArgs g = heads(d_ao, H, (long)R * H, d, Q + 2 * H, 3 * H, rowsH3, d, ws.dP, Rp, RR * nh, RR, R, R, d, 0, 1, 1.0f, causal ? 2 : 0);
        if ((rc = bgemm<float, T, MF>(g, n * nh, st))) return rc;
        g = heads(a.SP, Rp, RR * nh, RR, d_ao, H, (long)R * H, d, dqkv + 2 * H, 3 * H, rowsH3, d, R, d, R, 1, 0, 1.0f, 0);
        if ((rc = bgemm<float, float, MF>(g, n * nh, st))) return rc;
        attn_ds_kernel<<<(unsigned)(((size_t)n * nh * R + 3) / 4), 256, 0, st>>>(ws.dP, a.SP, (size_t)n * nh * R, R, Rp, full_from);
        if ((rc = vla_check_launch("attn_ds"))) return rc;
        g = heads(ws.dP, Rp, RR * nh, RR, Q + H, 3 * H, rowsH3, d, dqkv, 3 * H, rowsH3, d, R, d, R, 0, 0, isd, causal ? 1 : 0);
        if ((rc = bgemm<float, T, MF>(g, n * nh, st))) return rc;
        g = heads(ws.dP, Rp, RR * nh, RR, Q, 3 * H, rowsH3, d, dqkv + H, 3 * H, rowsH3, d, R, d, R, 1, 0, isd, 0);
        if ((rc = bgemm<float, T, MF>(g, n * nh, st))) return rc;
        rope_rows_kernel<T><<<blocks_for((size_t)M * 3 * (H / 2)), 256, 0, st>>>((T *)ws.dQKVb, dqkv, ws.rope, (size_t)M, R, H, d, -1.0f);
        if ((rc = vla_check_launch("rope_rows (transpose)"))) return rc;
        // ---- Q / K / V projections and the attention norm
        if ((rc = lora_group(group_of(3, &lo.q, &gr.q, H, H), a.Nrm, ws.dQKVb, first))) return rc;       // q, k, v adjacent
        if ((rc = transpose(lw.wq, H, H, 3 * H, 0)) || (rc = transpose(lw.wk, H, H, 3 * H, H)) || (rc = transpose(lw.wv, H, H, 3 * H, 2 * H))) return rc;
        if ((rc = gemm(ws.dQKVb, ws.Wt, nullptr, nullptr, 1, H, a.GU, 3 * H))) return rc;      // d n [M, H]
        rmsnorm_bwd_kernel<T><<<M, 256, 0, st>>>(ws.dX, (T *)ws.dXb, a.x_in, (const float *)lw.attn_norm, a.GU, H, c.rms_eps);
        return vla_check_launch("rmsnorm_bwd");
    }
};

template <typename T>
int backward_impl(vla_model *m, void *wsbuf, bool keep, const void *patch, const int32_t *ids, const int32_t *bins, const float *coef, int N,
                  int P, int T_, int A, int mode, const void *slot_embed, float temperature, int rank, float scale,
                  const vla_lora_layer *lora, const vla_lora_layer_grads *grads, float *logp, hipStream_t st) {
    const vla_config &c = m->cfg;
    const int S = P + T_, H = c.hidden, L = c.n_layers;
    const int R = (mode == VLA_MODE_AR) ? S + A - 1 : S + A;
    const int first_row = (mode == VLA_MODE_AR) ? S - 1 : S;
    const int mb = bw_micro_batch(c, N);
    const T *head = (const T *)m->w.lm_head + (size_t)(c.vocab - VLA_N_BINS) * H;
    int rc;
    Backward<T> bw{m, c, plan_bw(c, (char *)wsbuf, mb, R, rank, keep), st, 0, R, 0, H, c.ffn, H / c.n_heads, c.n_heads,
                   mode == VLA_MODE_AR ? 0x7fffffff : S, rank, scale, mb};
    if ((rc = launch_rope_table(bw.ws.rope, R, 0, bw.d, c.rope_theta, st))) return rc;
    bool first = true;
    for (int n0 = 0; n0 < N; n0 += mb, first = false) {
        const int n = (N - n0 < mb) ? N - n0 : mb;
        bw.n = n; bw.M = n * R;
        const size_t MH = (size_t)bw.M * H;
        const T *pp = patch ? (const T *)patch + (size_t)n0 * P * H : nullptr;
        const int32_t *ii = ids ? ids + (size_t)n0 * T_ : nullptr;
        const float *x_final = nullptr;
        if (keep) {
            // (1) forward with the unfused kernels, every layer leaving what its backward reads in a set of its own
            if ((rc = launch_embed_prefix<T>(bw.ws.X, pp, ii, (const T *)m->w.embed, n, P, T_, R, H, c.vocab, st))) return rc;
            if (mode == VLA_MODE_AR) {
                if ((rc = launch_embed_tokens<T>(bw.ws.X, bins + (size_t)n0 * A, A, A - 1, (const T *)m->w.embed, n, R, S, H, c.vocab, st))) return rc;
            } else if ((rc = launch_embed_slots<T>(bw.ws.X, (const T *)slot_embed, n, A, R, S, H, st))) return rc;
            for (int l = 0; l < L; l++)
                if ((rc = bw.layer_forward(l, bw.acts(l), true))) return rc;
            x_final = bw.ws.X;
        } else {
            // (1) the forward pass of the recompute itself (its fused kernels), keeping every layer's input
            if ((rc = vla_forward_streams(m, bw.ws.fw, mb, pp, ii, bins + (size_t)n0 * A, n, P, T_, A, mode, slot_embed, bw.ws.ckpt, &x_final, st))) return rc;
        }
        fill_kernel<<<blocks_for(MH), 256, 0, st>>>(bw.ws.dX, MH, 0.f);
        if ((rc = vla_check_launch("fill"))) return rc;
        head_bwd_kernel<T><<<n * A, 256, (size_t)(H + VLA_N_BINS) * sizeof(float), st>>>(
            bw.ws.dX, logp ? logp + (size_t)n0 * A : nullptr, x_final, (const float *)m->w.final_norm, head, bins + (size_t)n0 * A,
            coef + (size_t)n0 * A, A, R, first_row, H, c.rms_eps, 1.0f / temperature);
        if ((rc = vla_check_launch("head_bwd"))) return rc;
        if ((rc = bw.cast(bw.ws.dXb, bw.ws.dX, H, H, H))) return rc;
        for (int l = L - 1; l >= 0; l--)
            if ((rc = bw.layer_backward(l, lora[l], grads[l], first))) return rc;
    }
    return 0;
}

bool lora_layer_complete(const vla_lora_layer &l, const vla_lora_layer_grads &g) {
    const vla_lora_factor *f = &l.q;
    const vla_lora_grad *d = &g.q;
    for (int i = 0; i < 7; i++)
        if (!f[i].a || !f[i].b || !d[i].da || !d[i].db) return false;
    return true;
}

}  // namespace

extern "C" {

size_t vla_backward_workspace_bytes(const vla_config *cfg, int N, int S, int A, int rank) {
    if (vla_check_config(cfg)) return 0;
    if (N <= 0 || S <= 0 || A <= 0 || rank <= 0) { vla_set_error("N, S, A and rank must be positive"); return 0; }
    if (S + A > cfg->max_seq + 1) { vla_set_error("S + A exceeds capacity"); return 0; }
    const int R = (S + A <= cfg->max_seq) ? S + A : S + A - 1;
    return plan_bw(*cfg, nullptr, bw_micro_batch(*cfg, N), R, rank, false).total;
}

size_t vla_backward_keep_workspace_bytes(const vla_config *cfg, int N, int S, int A, int rank) {
    if (vla_check_config(cfg)) return 0;
    if (N <= 0 || S <= 0 || A <= 0 || rank <= 0) { vla_set_error("N, S, A and rank must be positive"); return 0; }
    if (S + A > cfg->max_seq + 1) { vla_set_error("S + A exceeds capacity"); return 0; }
    const int R = (S + A <= cfg->max_seq) ? S + A : S + A - 1;
    return plan_bw(*cfg, nullptr, bw_micro_batch(*cfg, N), R, rank, true).total;
}

int vla_logprob_backward(vla_model *m, void *ws, size_t ws_bytes, const void *patch, const int32_t *ids, const int32_t *bins,
                         const float *coef, int N, int P, int T, int A, int mode, const void *slot_embed, float temperature,
                         int rank, float scale, int keep_activations, const vla_lora_layer *lora,
                         const vla_lora_layer_grads *grads, float *logp, void *stream) {
    if (!m || !ws || !bins || !coef || !lora || !grads) { vla_set_error("model, ws, bins, coef, lora or grads is NULL"); return VLA_EINVAL; }
    if (mode != VLA_MODE_AR && mode != VLA_MODE_PARALLEL_CHUNK) { vla_set_error("unknown mode %d", mode); return VLA_EINVAL; }
    if (N <= 0 || P < 0 || T < 0 || P + T < 1 || A <= 0 || rank <= 0) { vla_set_error("need N, A, rank >= 1, P, T >= 0, P + T >= 1"); return VLA_EINVAL; }
    if ((P > 0 && !patch) || (T > 0 && !ids)) { vla_set_error("patch / ids is NULL"); return VLA_EINVAL; }
    if (!(temperature > 0.f)) { vla_set_error("temperature must be positive"); return VLA_EINVAL; }
    if (mode == VLA_MODE_PARALLEL_CHUNK && !slot_embed) { vla_set_error("slot_embed is NULL"); return VLA_EINVAL; }
    const vla_config &c = m->cfg;
    for (int l = 0; l < c.n_layers; l++)
        if (!lora_layer_complete(lora[l], grads[l])) { vla_set_error("layer %d has a NULL LoRA factor or gradient pointer", l); return VLA_EINVAL; }
    const int S = P + T, R = (mode == VLA_MODE_AR) ? S + A - 1 : S + A;
    if (R > c.max_seq) { vla_set_error("rows per rollout %d exceed max_seq %d", R, c.max_seq); return VLA_ESHAPE; }
    const int mb = bw_micro_batch(c, N);
    if ((size_t)mb * R * (size_t)(c.ffn > 3 * c.hidden ? 2 * c.ffn : 3 * c.hidden) * 4 >= ((size_t)1 << 40)) { vla_set_error("micro-batch too large"); return VLA_ESHAPE; }
    if (3 * rank > 256) { vla_set_error("rank %d unsupported (at most 85: three stacked factors fill 256 rows)", rank); return VLA_ESHAPE; }
    if (int rc = vla_check_rows_per_pass(c, mb, R)) return rc;
    const bool keep = keep_activations != 0;
    const size_t need = plan_bw(c, nullptr, mb, R, rank, keep).total;
    if (ws_bytes < need) { vla_set_error("workspace %zu bytes, need %zu", ws_bytes, need); return VLA_EWORKSPACE; }
    hipStream_t st = (hipStream_t)stream;
    return c.dtype == VLA_DTYPE_F32
               ? backward_impl<float>(m, ws, keep, patch, ids, bins, coef, N, P, T, A, mode, slot_embed, temperature, rank, scale, lora, grads, logp, st)
               : backward_impl<bf16_t>(m, ws, keep, patch, ids, bins, coef, N, P, T, A, mode, slot_embed, temperature, rank, scale, lora, grads, logp, st);
}

}  // extern "C"
