// Shape-generic kernels of libvla: every step of the rollout / recompute path for any supported
// dimensions, with fp32 or bf16 storage (fp32 arithmetic throughout).  The tiny fp32 workload
// runs entirely on these; the bf16 7B-shape workloads replace the GEMMs and the attention by the
// MFMA / streaming kernels of the other translation units and keep the rest.
#include "vla_internal.h"

namespace {

__device__ __forceinline__ float to_f(float v) { return v; }
__device__ __forceinline__ float to_f(bf16_t v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f(float v);
template <> __device__ __forceinline__ float from_f<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f<bf16_t>(float v) { return (bf16_t)v; }

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

// Sum over a 256-thread block; `red` is 4 floats of LDS.  Every thread gets the total.
__device__ __forceinline__ float block_sum_256(float v, float *red) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return red[0] + red[1] + red[2] + red[3];
}

// ---------------------------------------------------------------------------------- embedding
// Prefix assembly: x_p = patch[p] (p < P), x_{P+t} = embed[ids[t]].
template <typename T>
__global__ void embed_prefix_kernel(float *X, const T *patch, const int32_t *ids, const T *embed, int P,
                                    int T_, int rows_per_seq, int H, int vocab) {
    int S = P + T_;
    int s = blockIdx.x / S, p = blockIdx.x % S;
    const T *src;
    if (p < P) {
        src = patch + ((size_t)s * P + p) * H;
    } else {
        int id = ids[(size_t)s * T_ + (p - P)];
        id = min(max(id, 0), vocab - 1);
        src = embed + (size_t)id * H;
    }
    float *dst = X + ((size_t)s * rows_per_seq + p) * H;
    for (int i = threadIdx.x; i < H; i += blockDim.x) dst[i] = to_f(src[i]);
}

// Stored action tokens (teacher forcing): row row0 + j of sequence s is embed[vocab-256+bins[s][j]].
template <typename T>
__global__ void embed_tokens_kernel(float *X, const int32_t *bins, int bins_stride, int n_tok,
                                    const T *embed, int rows_per_seq, int row0, int H, int vocab) {
    int s = blockIdx.x / n_tok, j = blockIdx.x % n_tok;
    int b = bins[(size_t)s * bins_stride + j];
    b = min(max(b, 0), VLA_N_BINS - 1);
    const T *src = embed + (size_t)(vocab - VLA_N_BINS + b) * H;
    float *dst = X + ((size_t)s * rows_per_seq + row0 + j) * H;
    for (int i = threadIdx.x; i < H; i += blockDim.x) dst[i] = to_f(src[i]);
}

template <typename T>
__global__ void embed_slots_kernel(float *X, const T *slot_embed, int A, int rows_per_seq, int row0, int H) {
    int s = blockIdx.x / A, a = blockIdx.x % A;
    const T *src = slot_embed + (size_t)a * H;
    float *dst = X + ((size_t)s * rows_per_seq + row0 + a) * H;
    for (int i = threadIdx.x; i < H; i += blockDim.x) dst[i] = to_f(src[i]);
}

// ---------------------------------------------------------------------------------- RMSNorm
// n_i = x_i / sqrt(mean(x^2) + eps) * g_i; one 256-thread block per row.
template <typename T>
__global__ void rmsnorm_kernel(T *out, const float *X, const float *gain, int H, float eps) {
    __shared__ float red[4];
    const float *x = X + (size_t)blockIdx.x * H;
    float ss = 0.f;
    for (int i = threadIdx.x; i < H; i += 256) ss += x[i] * x[i];
    ss = block_sum_256(ss, red);
    float r = 1.0f / sqrtf(ss / (float)H + eps);
    T *o = out + (size_t)blockIdx.x * H;
    for (int i = threadIdx.x; i < H; i += 256) o[i] = from_f<T>(x[i] * r * gain[i]);
}

// Final norm of selected rows: out row (s * n_rows + j) = norm(X[s * rows_per_seq + row0 + j]).
__global__ void final_norm_rows_kernel(float *out, const float *X, const float *gain, int rows_per_seq,
                                       int row0, int n_rows, int H, float eps) {
    __shared__ float red[4];
    int s = blockIdx.x / n_rows, j = blockIdx.x % n_rows;
    const float *x = X + ((size_t)s * rows_per_seq + row0 + j) * H;
    float ss = 0.f;
    for (int i = threadIdx.x; i < H; i += 256) ss += x[i] * x[i];
    ss = block_sum_256(ss, red);
    float r = 1.0f / sqrtf(ss / (float)H + eps);
    float *o = out + (size_t)blockIdx.x * H;
    for (int i = threadIdx.x; i < H; i += 256) o[i] = x[i] * r * gain[i];
}

// ---------------------------------------------------------------------------------- GEMM
// C[M, N] = A[M, K] . W^T with W given as n_seg row blocks [segN, K].  64 x 64 output tile per
// 256-thread block, 4 x 4 outputs per thread, K stepped by 16 through LDS; every load and store is
// bounds checked.  EPI_SWIGLU computes silu(A.Wg^T) * (A.Wu^T) with both products in one pass.
template <typename T, int EPI>
__global__ void __launch_bounds__(256) gemm_generic_kernel(const T *A, const T *W0, const T *W1,
                                                           const T *W2, int segN, void *Cv, int M, int N,
                                                           int K) {
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ float As[BK][BM + 1];
    __shared__ float Ws[BK][BN + 1];
    __shared__ float Us[(EPI == EPI_SWIGLU) ? BK : 1][BN + 1];
    int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    float acc[4][4] = {}, acu[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += BK) {
        for (int e = threadIdx.x; e < BM * BK; e += 256) {
            int r = e / BK, kk = e % BK;
            int m = m0 + r, k = k0 + kk;
            As[kk][r] = (m < M && k < K) ? to_f(A[(size_t)m * K + k]) : 0.f;
            int n = n0 + r;
            float w = 0.f, u = 0.f;
            if (n < N && k < K) {
                if (EPI == EPI_SWIGLU) {
                    w = to_f(W0[(size_t)n * K + k]);
                    u = to_f(W1[(size_t)n * K + k]);
                } else {
                    int seg = n / segN, nn = n % segN;
                    const T *Wp = seg == 0 ? W0 : (seg == 1 ? W1 : W2);
                    w = to_f(Wp[(size_t)nn * K + k]);
                }
            }
            Ws[kk][r] = w;
            if (EPI == EPI_SWIGLU) Us[kk][r] = u;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; kk++) {
            float a[4], w[4], u[4];
#pragma unroll
            for (int i = 0; i < 4; i++) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; j++) w[j] = Ws[kk][tx * 4 + j];
            if (EPI == EPI_SWIGLU) {
#pragma unroll
                for (int j = 0; j < 4; j++) u[j] = Us[kk][tx * 4 + j];
            }
#pragma unroll
            for (int i = 0; i < 4; i++)
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    acc[i][j] += a[i] * w[j];
                    if (EPI == EPI_SWIGLU) acu[i][j] += a[i] * u[j];
                }
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; i++) {
        int m = m0 + ty * 4 + i;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            size_t o = (size_t)m * N + n;
            if (EPI == EPI_RESIDUAL) {
                ((float *)Cv)[o] += acc[i][j];
            } else if (EPI == EPI_SWIGLU) {
                float g = acc[i][j];
                ((T *)Cv)[o] = from_f<T>(g / (1.0f + expf(-g)) * acu[i][j]);
            } else {
                ((float *)Cv)[o] = acc[i][j];
            }
        }
    }
}

// ---------------------------------------------------------------------------------- rotary
// table[r][i] = (cos, sin)(phi), phi = (pos0 + r) * theta^(-2i/d), evaluated in fp64.
__global__ void rope_table_kernel(float2 *table, int R, int pos0, int d, float theta) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    int half = d / 2;
    if (idx >= R * half) return;
    int r = idx / half, i = idx % half;
    double inv = pow((double)theta, -2.0 * (double)i / (double)d);
    double phi = (double)(pos0 + r) * inv;
    table[idx] = make_float2((float)cos(phi), (float)sin(phi));
}

// Rotate q and k of every new row (pairs (i, i + d/2)) from the fp32 QKV projection, write q to its
// own [M, H] buffer and k, v into the KV layout.  One thread per (row, head, 8-dim chunk c of the first
// half): it owns dims [8c, 8c+8) and [d/2 + 8c, d/2 + 8c + 8).
template <typename T>
__global__ void rope_kv_write_kernel(T *q_out, const float *qkv, const float2 *table, T *kc, T *vc, int n_seq,
                                     int R, int pos0, int n_heads, int d, int pos_stride, int H) {
    int chunks = d / 16;
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)n_seq * R * n_heads * chunks;
    if (idx >= total) return;
    int c = idx % chunks;
    int h = (idx / chunks) % n_heads;
    size_t m = idx / ((size_t)chunks * n_heads);
    int s = m / R, r = m % R;
    int pos = pos0 + r;
    int half = d / 2;
    const float *q = qkv + m * 3 * (size_t)H + (size_t)h * d;
    const float *k = q + H;
    const float *v = q + 2 * (size_t)H;
    T *qo = q_out + m * (size_t)H + (size_t)h * d;
    size_t head = (size_t)s * n_heads + h;
    T *kdst_lo = kc + ((head * (d / 8) + c) * pos_stride + pos) * 8;
    T *kdst_hi = kc + ((head * (d / 8) + (half / 8) + c) * pos_stride + pos) * 8;
    T *vdst = vc + (head * pos_stride + pos) * d;
#pragma unroll
    for (int e = 0; e < 8; e++) {
        int i = c * 8 + e;
        float2 cs = table[(size_t)r * half + i];
        float qa = q[i], qb = q[i + half];
        float ka = k[i], kb = k[i + half];
        qo[i] = from_f<T>(qa * cs.x - qb * cs.y);
        qo[i + half] = from_f<T>(qb * cs.x + qa * cs.y);
        kdst_lo[e] = from_f<T>(ka * cs.x - kb * cs.y);
        kdst_hi[e] = from_f<T>(kb * cs.x + ka * cs.y);
        vdst[i] = from_f<T>(v[i]);
        vdst[i + half] = from_f<T>(v[i + half]);
    }
}

// Rows first .. first + count - 1 of every sequence of X [n_seq * R, H], packed into Xt [n_seq * count, H].
__global__ void gather_rows_kernel(float *Xt, const float *X, int R, int first, int count, int H) {
    const int s = blockIdx.x / count, j = blockIdx.x - s * count;
    const f32x4_t *src = (const f32x4_t *)(X + ((size_t)s * R + first + j) * H);
    f32x4_t *dst = (f32x4_t *)(Xt + (size_t)blockIdx.x * H);
    for (int i = threadIdx.x; i < H / 4; i += blockDim.x) dst[i] = src[i];
}

// Rotary on q alone: qf fp32 [M, H] (row m of sequence s is position table row first + m % count) -> q_out in the
// storage type.  One thread per (row, head, pair index).
template <typename T>
__global__ void rope_q_kernel(T *q_out, const float *qf, const float2 *table, size_t M, int count, int first, int n_heads,
                              int d, int H) {
    const int half = d / 2;
    const size_t total = M * (size_t)n_heads * half;
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int i = (int)(idx % half);
    const int h = (int)((idx / half) % n_heads);
    const size_t m = idx / ((size_t)half * n_heads);
    const float2 cs = table[(size_t)(first + (int)(m % count)) * half + i];
    const size_t o = m * (size_t)H + (size_t)h * d + i;
    const float a = qf[o], b = qf[o + half];
    q_out[o] = from_f<T>(a * cs.x - b * cs.y);
    q_out[o + half] = from_f<T>(b * cs.x + a * cs.y);
}

// ---------------------------------------------------------------------------------- attention
// One wave per (sequence, head, new row): scores over the allowed keys into LDS, softmax, then
// the weighted sum of V rows with each lane owning head dims lane, lane+64, ...
template <typename T>
__global__ void __launch_bounds__(256) attention_generic_kernel(T *out, const T *qbuf, const T *kc,
                                                               const T *vc, int n_seq, int R, int pos0,
                                                               int full_from, int n_heads, int d,
                                                               int pos_stride, int H) {
    extern __shared__ float smem[];
    int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n_keys = pos0 + R;            // the most keys any row of this launch sees
    int per_wave = n_keys + d;
    float *sc = smem + (size_t)wave * per_wave;
    float *qs = sc + n_keys;
    size_t item = (size_t)blockIdx.x * 4 + wave;
    size_t total = (size_t)n_seq * n_heads * R;
    if (item >= total) return;      // whole wave leaves together; no block-level barrier below
    int r = item % R;
    int h = (item / R) % n_heads;
    int s = item / ((size_t)R * n_heads);
    size_t m = (size_t)s * R + r;
    int pos = pos0 + r;
    int nk = (pos >= full_from) ? (pos0 + R) : (pos + 1);
    const T *q = qbuf + m * (size_t)H + (size_t)h * d;
    for (int i = lane; i < d; i += 64) qs[i] = to_f(q[i]);
    __builtin_amdgcn_wave_barrier();
    size_t head = (size_t)s * n_heads + h;
    const T *kh = kc + head * (size_t)d * pos_stride;
    const T *vh = vc + head * (size_t)pos_stride * d;
    float scale = 1.0f / sqrtf((float)d);
    float mx = -INFINITY;
    for (int p = lane; p < nk; p += 64) {
        float acc = 0.f;
        for (int c = 0; c < d / 8; c++) {
            const T *kp = kh + ((size_t)c * pos_stride + p) * 8;
#pragma unroll
            for (int e = 0; e < 8; e++) acc += qs[c * 8 + e] * to_f(kp[e]);
        }
        acc *= scale;
        sc[p] = acc;
        mx = fmaxf(mx, acc);
    }
    mx = wave_max(mx);
    float sum = 0.f;
    for (int p = lane; p < nk; p += 64) {
        float e = expf(sc[p] - mx);
        sc[p] = e;
        sum += e;
    }
    sum = wave_sum(sum);
    __builtin_amdgcn_wave_barrier();
    float inv = 1.0f / sum;
    for (int i = lane; i < d; i += 64) {
        float acc = 0.f;
        for (int p = 0; p < nk; p++) acc += sc[p] * to_f(vh[(size_t)p * d + i]);
        out[m * (size_t)H + (size_t)h * d + i] = from_f<T>(acc * inv);
    }
}

// ---------------------------------------------------------------------------------- head + sampler
// One 256-thread block per row.  Logits over the 256 action bins (one bin per thread), then wave 0
// reduces the softmax statistics and the Gumbel-max choice with four bins per lane (bins lane, lane+64, +128, +192).
template <typename T>
__global__ void __launch_bounds__(256) head_sample_kernel(const float *h, const T *Wb, int H, float temperature,
                                                         const float *gumbel, const int32_t *given,
                                                         int32_t *bins_out, float *logp, float *ent,
                                                         float *logits, int out_stride, int out_off,
                                                         float *X_next, const T *embed, int vocab) {
    extern __shared__ float smem[];
    float *hs = smem;               // [H]
    float *z = smem + H;            // [256]
    __shared__ int chosen;
    int row = blockIdx.x;
    size_t o = (size_t)row * out_stride + out_off;
    int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float *hr = h + (size_t)row * H;
    for (int i = threadIdx.x; i < H; i += 256) hs[i] = hr[i];
    __syncthreads();
    {   // thread k owns bin k: its weight row is walked in 16-byte pieces, h is broadcast from LDS
        const int k = threadIdx.x;
        const T *w = Wb + (size_t)k * H;
        constexpr int V = 16 / sizeof(T);
        float a0 = 0.f, a1 = 0.f;
        int i = 0;
        if (H % V == 0) {
            typedef T vec_t __attribute__((ext_vector_type(V)));
            for (; i + 2 * V <= H; i += 2 * V) {
                vec_t w0 = *(const vec_t *)(w + i), w1 = *(const vec_t *)(w + i + V);
#pragma unroll
                for (int e = 0; e < V; e++) { a0 += hs[i + e] * to_f(w0[e]); a1 += hs[i + V + e] * to_f(w1[e]); }
            }
        }
        for (; i < H; i++) a0 += hs[i] * to_f(w[i]);
        z[k] = a0 + a1;
    }
    __syncthreads();
    if (logits) logits[o * VLA_N_BINS + threadIdx.x] = z[threadIdx.x];
    if (wave == 0) {
        float y[4], t[4];
        float mx = -INFINITY;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            int k = lane + 64 * j;
            y[j] = z[k] / temperature;
            t[j] = gumbel ? y[j] + gumbel[o * VLA_N_BINS + k] : y[j];
            mx = fmaxf(mx, y[j]);
        }
        mx = wave_max(mx);
        float se = 0.f, sy = 0.f;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            float e = expf(y[j] - mx);
            se += e;
            sy += e * y[j];
        }
        se = wave_sum(se);
        sy = wave_sum(sy);
        float lse = mx + logf(se);
        // argmax of t, lowest bin index on ties
        float bt = t[0];
        int bk = lane;
#pragma unroll
        for (int j = 1; j < 4; j++)
            if (t[j] > bt) { bt = t[j]; bk = lane + 64 * j; }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            float ot = __shfl_xor(bt, off, 64);
            int ok = __shfl_xor(bk, off, 64);
            if (ot > bt || (ot == bt && ok < bk)) { bt = ot; bk = ok; }
        }
        int bin = bk;
        if (given) bin = min(max(given[o], 0), VLA_N_BINS - 1);
        if (lane == 0) {
            if (bins_out) bins_out[o] = bin;
            logp[o] = z[bin] / temperature - lse;
            ent[o] = lse - sy / se;
            chosen = bin;
        }
    }
    if (X_next) {
        __syncthreads();
        const T *src = embed + (size_t)(vocab - VLA_N_BINS + chosen) * H;
        float *dst = X_next + (size_t)row * H;
        for (int i = threadIdx.x; i < H; i += 256) dst[i] = to_f(src[i]);
    }
}

// value[row, c] = w[c] . h[row] + b + bias[c]; one workgroup per (row, c).
__global__ void value_head_kernel(float *value, const float *h, const float *w, float b, const float *bias, int H,
                                  int h_stride) {
    __shared__ float red[4];
    const int c = blockIdx.y, vd = gridDim.y;
    const float *hr = h + (size_t)blockIdx.x * h_stride, *wc = w + (size_t)c * H;
    float acc = 0.f;
    for (int i = threadIdx.x; i < H; i += 256) acc += hr[i] * wc[i];
    acc = block_sum_256(acc, red);
    if (threadIdx.x == 0) value[(size_t)blockIdx.x * vd + c] = acc + b + (bias ? bias[c] : 0.f);
}

}  // namespace

// =========================================================================================== host
template <typename T>
int launch_embed_prefix(float *X, const T *patch, const int32_t *ids, const T *embed, int n_seq, int P,
                        int T_, int rows_per_seq, int H, int vocab, hipStream_t st) {
    if (n_seq * (P + T_) == 0) return 0;
    ProfScope ps("embed_prefix", 0.0, st);
    embed_prefix_kernel<T><<<n_seq * (P + T_), 256, 0, st>>>(X, patch, ids, embed, P, T_, rows_per_seq, H, vocab);
    return vla_check_launch("embed_prefix");
}
template <typename T>
int launch_embed_tokens(float *X, const int32_t *bins, int bins_stride, int n_tok, const T *embed,
                        int n_seq, int rows_per_seq, int row0, int H, int vocab, hipStream_t st) {
    if (n_seq * n_tok == 0) return 0;
    ProfScope ps("embed_tokens", 0.0, st);
    embed_tokens_kernel<T><<<n_seq * n_tok, 256, 0, st>>>(X, bins, bins_stride, n_tok, embed, rows_per_seq, row0, H, vocab);
    return vla_check_launch("embed_tokens");
}
template <typename T>
int launch_embed_slots(float *X, const T *slot_embed, int n_seq, int A, int rows_per_seq, int row0,
                       int H, hipStream_t st) {
    if (n_seq * A == 0) return 0;
    ProfScope ps("embed_slots", 0.0, st);
    embed_slots_kernel<T><<<n_seq * A, 256, 0, st>>>(X, slot_embed, A, rows_per_seq, row0, H);
    return vla_check_launch("embed_slots");
}
template <typename T>
int launch_rmsnorm(T *out, const float *X, const float *gain, int M, int H, float eps, hipStream_t st) {
    if (M == 0) return 0;
    ProfScope ps("rmsnorm", (double)M * H * (4 + sizeof(T)), st);
    rmsnorm_kernel<T><<<M, 256, 0, st>>>(out, X, gain, H, eps);
    return vla_check_launch("rmsnorm");
}
int launch_final_norm_rows(float *out, const float *X, const float *gain, int n_seq, int rows_per_seq,
                           int row0, int n_rows, int H, float eps, hipStream_t st) {
    if (n_seq * n_rows == 0) return 0;
    ProfScope ps("final_norm_rows", 0.0, st);
    final_norm_rows_kernel<<<n_seq * n_rows, 256, 0, st>>>(out, X, gain, rows_per_seq, row0, n_rows, H, eps);
    return vla_check_launch("final_norm_rows");
}
template <typename T>
int launch_gemm_generic(const GemmArgs &g, hipStream_t st) {
    if (g.M == 0) return 0;
    ProfScope ps("gemm_generic", 2.0 * g.M * g.K * g.n_seg * g.segN, st);
    int N = (g.epilogue == EPI_SWIGLU) ? g.segN : g.n_seg * g.segN;
    dim3 grid((N + 63) / 64, (g.M + 63) / 64);
    const T *A = (const T *)g.A, *W0 = (const T *)g.W[0], *W1 = (const T *)g.W[1], *W2 = (const T *)g.W[2];
    if (g.epilogue == EPI_STORE)
        gemm_generic_kernel<T, EPI_STORE><<<grid, 256, 0, st>>>(A, W0, W1, W2, g.segN, g.C, g.M, N, g.K);
    else if (g.epilogue == EPI_RESIDUAL)
        gemm_generic_kernel<T, EPI_RESIDUAL><<<grid, 256, 0, st>>>(A, W0, W1, W2, g.segN, g.C, g.M, N, g.K);
    else
        gemm_generic_kernel<T, EPI_SWIGLU><<<grid, 256, 0, st>>>(A, W0, W1, W2, g.segN, g.C, g.M, N, g.K);
    return vla_check_launch("gemm_generic");
}
int launch_rope_table(float2 *table, int R, int pos0, int d, float theta, hipStream_t st) {
    ProfScope ps("rope_table", 0.0, st);
    int n = R * (d / 2);
    if (n == 0) return 0;
    rope_table_kernel<<<(n + 255) / 256, 256, 0, st>>>(table, R, pos0, d, theta);
    return vla_check_launch("rope_table");
}
template <typename T>
int launch_rope_kv_write(T *q_out, const float *qkv, const float2 *table, const KvView &kv, int layer,
                         const RowsArgs &ra, int H, hipStream_t st) {
    ProfScope ps("rope_kv_write", (double)ra.n_seq * ra.R * H * 5 * sizeof(T), st);
    size_t total = (size_t)ra.n_seq * ra.R * kv.n_heads * (kv.d / 16);
    if (total == 0) return 0;
    T *kc = (T *)kv.k + (size_t)layer * kv.layer_elems;
    T *vc = (T *)kv.v + (size_t)layer * kv.layer_elems;
    rope_kv_write_kernel<T><<<(unsigned)((total + 255) / 256), 256, 0, st>>>(
        q_out, qkv, table, kc, vc, ra.n_seq, ra.R, ra.pos0, kv.n_heads, kv.d, kv.pos_stride, H);
    return vla_check_launch("rope_kv_write");
}
int launch_gather_rows(float *Xt, const float *X, int n_seq, int R, int first, int count, int H, hipStream_t st) {
    if (n_seq * count == 0) return 0;
    ProfScope ps("gather_rows", 0.0, st);
    gather_rows_kernel<<<n_seq * count, 256, 0, st>>>(Xt, X, R, first, count, H);
    return vla_check_launch("gather_rows");
}
template <typename T>
int launch_rope_q(T *q_out, const float *qf, const float2 *table, int n_seq, int count, int first, int n_heads, int d, int H,
                  hipStream_t st) {
    const size_t M = (size_t)n_seq * count, total = M * n_heads * (d / 2);
    if (total == 0) return 0;
    ProfScope ps("rope_q", 0.0, st);
    rope_q_kernel<T><<<(unsigned)((total + 255) / 256), 256, 0, st>>>(q_out, qf, table, M, count, first, n_heads, d, H);
    return vla_check_launch("rope_q");
}
template <typename T>
int launch_attention_generic(T *out, const T *q, const KvView &kv, int layer, const RowsArgs &ra,
                             int H, hipStream_t st) {
    ProfScope ps("attention_generic", 0.0, st);
    size_t total = (size_t)ra.n_seq * kv.n_heads * ra.R;
    if (total == 0) return 0;
    const T *kc = (const T *)kv.k + (size_t)layer * kv.layer_elems;
    const T *vc = (const T *)kv.v + (size_t)layer * kv.layer_elems;
    // scores of the visible keys + the query, per wave; above the 64 KB default the limit is raised once per
    // instantiation (8192 keys at head_dim 256 need 132 KB of the CU's 160 KB)
    size_t lds = (size_t)4 * (ra.pos0 + ra.R + kv.d) * sizeof(float);
    if (lds > 64 * 1024) {
        static bool raised = false;
        if (lds > 160 * 1024) { vla_set_error("attention_generic: %d keys need %zu bytes of LDS", ra.pos0 + ra.R, lds); return VLA_ESHAPE; }
        if (!raised) {
            if (hipFuncSetAttribute((const void *)attention_generic_kernel<T>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    160 * 1024) != hipSuccess) {
                vla_set_error("attention_generic: cannot raise the dynamic LDS limit");
                return VLA_EHIP;
            }
            raised = true;
        }
    }
    attention_generic_kernel<T><<<(unsigned)((total + 3) / 4), 256, lds, st>>>(
        out, q, kc, vc, ra.n_seq, ra.R, ra.pos0, ra.full_from, kv.n_heads, kv.d, kv.pos_stride, H);
    return vla_check_launch("attention_generic");
}
template <typename T>
int launch_head_sample(const float *h, const T *lm_head_bins, int n_rows, int H, float temperature,
                       const float *gumbel, const int32_t *given_bins, int32_t *bins_out, float *logp,
                       float *ent, float *logits, int out_stride, int out_off, float *X_next,
                       const T *embed, int vocab, hipStream_t st) {
    if (n_rows == 0) return 0;
    ProfScope ps("head_sample", 2.0 * n_rows * H * VLA_N_BINS, st);
    size_t lds = (size_t)(H + VLA_N_BINS) * sizeof(float);
    head_sample_kernel<T><<<n_rows, 256, lds, st>>>(h, lm_head_bins, H, temperature, gumbel, given_bins,
                                                    bins_out, logp, ent, logits, out_stride, out_off,
                                                    X_next, embed, vocab);
    return vla_check_launch("head_sample");
}
int launch_value_head(float *value, const float *h, const float *w, float b, const float *bias, int vd, int n,
                      int H, int h_stride, hipStream_t st) {
    if (n == 0) return 0;
    ProfScope ps("value_head", 0.0, st);
    value_head_kernel<<<dim3(n, vd), 256, 0, st>>>(value, h, w, b, bias, H, h_stride);
    return vla_check_launch("value_head");
}

#define INSTANTIATE(T)                                                                                        \
    template int launch_embed_prefix<T>(float *, const T *, const int32_t *, const T *, int, int, int, int,   \
                                        int, int, hipStream_t);                                               \
    template int launch_embed_tokens<T>(float *, const int32_t *, int, int, const T *, int, int, int, int,    \
                                        int, hipStream_t);                                                    \
    template int launch_embed_slots<T>(float *, const T *, int, int, int, int, int, hipStream_t);             \
    template int launch_rmsnorm<T>(T *, const float *, const float *, int, int, float, hipStream_t);          \
    template int launch_gemm_generic<T>(const GemmArgs &, hipStream_t);                                       \
    template int launch_rope_kv_write<T>(T *, const float *, const float2 *, const KvView &, int,             \
                                         const RowsArgs &, int, hipStream_t);                                                        \
    template int launch_attention_generic<T>(T *, const T *, const KvView &, int, const RowsArgs &, int,      \
                                             hipStream_t);                                                    \
    template int launch_rope_q<T>(T *, const float *, const float2 *, int, int, int, int, int, int, hipStream_t); \
    template int launch_head_sample<T>(const float *, const T *, int, int, float, const float *,              \
                                       const int32_t *, int32_t *, float *, float *, float *, int, int,       \
                                       float *, const T *, int, hipStream_t);
INSTANTIATE(float)
INSTANTIATE(bf16_t)
