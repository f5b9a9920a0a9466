// Weight-streaming bf16 GEMM for the decode steps: C[M, N] = A[M, K] . W[N, K]^T with M <= 256
// (one row per environment).  Every weight byte is read from HBM exactly once, so the kernel is laid
// out around that stream:
//   - a wave owns 32 weight rows (plus the 32 matching "up" rows for the SwiGLU projection) and reads
//     them straight from global memory into MFMA row-operand registers: per 64-wide K tile a lane
//     loads 64 contiguous bytes of one row (two lanes cover a 128-byte line), k slot (half, e) of
//     k-step j holding k = 32*half + 8*j + e;
//   - the M activation rows of the K tile (at most 32 KB) are staged once per workgroup in LDS with
//     the same 16-byte-chunk swizzle as the large GEMM and serve as the column operand of all waves;
//   - the K range is split across workgroups (grid.y) when N alone gives too few workgroups to pull
//     8 TB/s; partial sums go to fp32 scratch and a second kernel adds them in a fixed order (no
//     atomics: results are bit-reproducible) and applies the epilogue.
#include <stdlib.h>

#include <type_traits>

#include "vla_internal.h"

namespace {

constexpr int BK = 64;

struct SkinnyParams {
    const bf16_t *A;
    const bf16_t *W0, *W1, *W2;
    void *C;            // final output (splits == 1) ...
    float *P;           // ... or partial sums [splits][M][N]
    int M, N, K, segN, splits;
};

__device__ __forceinline__ int swz(int row) { return (row >> 1) & 7; }

// MB: number of 32-row activation blocks (M <= 32 * MB).  NB: weight-row blocks per wave.
template <int MB, int EPI>
__global__ void __launch_bounds__(256) gemm_skinny_kernel(SkinnyParams p) {
    constexpr int NB = (EPI == EPI_SWIGLU) ? 2 : 1;
    constexpr int A_TILE = MB * 32 * BK * 2;          // bytes per LDS stage
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int col = lane & 31, hh = lane >> 5;
    const int K = p.K;
    const int ktiles = K / BK;
    const int kt0 = (int)((long)blockIdx.y * ktiles / p.splits);
    const int kt1 = (int)((long)(blockIdx.y + 1) * ktiles / p.splits);

    // ---- weight rows of this wave ---------------------------------------------------------------
    const bf16_t *wrow[NB];
    int n_out;                                         // first output column of this wave
    if (EPI == EPI_SWIGLU) {
        int f = blockIdx.x * 128 + wave * 32;
        wrow[0] = p.W0 + (size_t)(f + col) * K + hh * 32;
        wrow[NB - 1] = p.W1 + (size_t)(f + col) * K + hh * 32;
        n_out = f;
    } else {
        int n = blockIdx.x * 128 + wave * 32;
        int seg = n / p.segN;
        const bf16_t *Wp = seg == 0 ? p.W0 : (seg == 1 ? p.W1 : p.W2);
        wrow[0] = Wp + (size_t)(n - seg * p.segN + col) * K + hh * 32;
        n_out = n;
    }

    // ---- activation staging: MB * 256 chunks of 16 bytes per K tile, MB per thread ------------------
    const bf16_t *asrc[MB];
#pragma unroll
    for (int i = 0; i < MB; i++) {
        int q = i * 256 + t;
        int row = q >> 3, pc = q & 7;
        int c = pc ^ swz(row);
        asrc[i] = p.A + (size_t)min(row, p.M - 1) * K + c * 8;
    }
    int a_off[MB], a_sw[MB];
#pragma unroll
    for (int i = 0; i < MB; i++) {
        int row = i * 32 + col;
        a_off[i] = row * 128;
        a_sw[i] = swz(row);
    }

    f32x16_t acc[NB][MB];
#pragma unroll
    for (int b = 0; b < NB; b++)
#pragma unroll
        for (int i = 0; i < MB; i++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[b][i][r] = 0.f;

    bf16x8_t wreg[3][NB][4], areg[MB];
    auto wload = [&](int buf, int kt) {
#pragma unroll
        for (int b = 0; b < NB; b++)
#pragma unroll
            for (int j = 0; j < 4; j++) wreg[buf][b][j] = *(const bf16x8_t *)(wrow[b] + (size_t)kt * BK + j * 8);
    };
    auto aload = [&](int kt) {
#pragma unroll
        for (int i = 0; i < MB; i++) areg[i] = *(const bf16x8_t *)(asrc[i] + (size_t)kt * BK);
    };
    auto astore = [&](int s) {
#pragma unroll
        for (int i = 0; i < MB; i++) *(bf16x8_t *)(lds + s * A_TILE + (i * 256 + t) * 16) = areg[i];
    };

    // One K tile: prefetch the weights two tiles ahead (register sets rotate 0,1,2 with compile-time
    // indices), the activations one tile ahead (through registers into the other LDS stage).
    auto body = [&](auto ws_c, int kt) {
        constexpr int WS = decltype(ws_c)::value;
        constexpr int WS2 = (WS + 2) % 3;
        const int s = (kt - kt0) & 1;
        const bool more = kt + 1 < kt1;
        if (more) aload(kt + 1);
        if (kt + 2 < kt1) wload(WS2, kt + 2);
        const char *base = lds + s * A_TILE;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const int c = hh * 4 + j;
            bf16x8_t af[MB];
#pragma unroll
            for (int i = 0; i < MB; i++) af[i] = *(const bf16x8_t *)(base + a_off[i] + ((c ^ a_sw[i]) << 4));
#pragma unroll
            for (int b = 0; b < NB; b++)
#pragma unroll
                for (int i = 0; i < MB; i++)
                    acc[b][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wreg[WS][b][j], af[i], acc[b][i], 0, 0, 0);
        }
        if (more) astore(s ^ 1);
        __syncthreads();
    };
    if (kt0 < kt1) {
        aload(kt0);
        wload(0, kt0);
        if (kt0 + 1 < kt1) wload(1, kt0 + 1);
        astore(0);
        __syncthreads();
        for (int kt = kt0; kt < kt1; kt += 3) {
            body(std::integral_constant<int, 0>{}, kt);
            if (kt + 1 < kt1) body(std::integral_constant<int, 1>{}, kt + 1);
            if (kt + 2 < kt1) body(std::integral_constant<int, 2>{}, kt + 2);
        }
    }

    // ---- output: lane holds activation row i*32 + col and weight rows 8*(r/4) + 4*hh + r%4 ----------
    const int nquad = 4 * hh;
#pragma unroll
    for (int i = 0; i < MB; i++) {
        const int m = i * 32 + col;
        if (m >= p.M) continue;
        if (p.splits > 1) {
            // partial sums [split][M][NB * N]: gate at column f, up at column N + f
            float *out = p.P + ((size_t)blockIdx.y * p.M + m) * (NB * p.N) + n_out;
#pragma unroll
            for (int b = 0; b < NB; b++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    f32x4_t v;
#pragma unroll
                    for (int e = 0; e < 4; e++) v[e] = acc[b][i][g * 4 + e];
                    *(f32x4_t *)(out + (size_t)b * p.N + g * 8 + nquad) = v;
                }
        } else if (EPI == EPI_SWIGLU) {
            bf16_t *out = (bf16_t *)p.C + (size_t)m * p.N + n_out;
#pragma unroll
            for (int g = 0; g < 4; g++) {
                bf16x4_t o;
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    float gate = acc[0][i][g * 4 + e], up = acc[NB - 1][i][g * 4 + e];
                    o[e] = (bf16_t)vla_silu_mul(gate, up);
                }
                *(bf16x4_t *)(out + g * 8 + nquad) = o;
            }
        } else if (EPI == EPI_RESIDUAL) {
            float *out = (float *)p.C + (size_t)m * p.N + n_out;
#pragma unroll
            for (int g = 0; g < 4; g++) {
                f32x4_t *dst = (f32x4_t *)(out + g * 8 + nquad);
                f32x4_t v = *dst;
#pragma unroll
                for (int e = 0; e < 4; e++) v[e] += acc[0][i][g * 4 + e];
                *dst = v;
            }
        } else {
            float *out = (float *)p.C + (size_t)m * p.N + n_out;
#pragma unroll
            for (int g = 0; g < 4; g++) {
                f32x4_t v;
#pragma unroll
                for (int e = 0; e < 4; e++) v[e] = acc[0][i][g * 4 + e];
                *(f32x4_t *)(out + g * 8 + nquad) = v;
            }
        }
    }
}

// Sum of the split-K partials in split order, then the epilogue.  One thread per four columns of
// one row; P is [splits][M][NP] with NP = N (or 2N for SwiGLU: gate columns then up columns).
template <int EPI>
__global__ void skinny_reduce_kernel(void *C, const float *P, int splits, int M, int N) {
    const int NP = (EPI == EPI_SWIGLU) ? 2 * N : N;
    size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i >= (size_t)M * N) return;
    const size_t m = i / N, n = i - m * N;
    const float *src = P + m * NP + n;
    f32x4_t s = *(const f32x4_t *)src, u = {0.f, 0.f, 0.f, 0.f};
    if (EPI == EPI_SWIGLU) u = *(const f32x4_t *)(src + N);
    for (int k = 1; k < splits; k++) {
        const float *sk = src + (size_t)k * M * NP;
        f32x4_t v = *(const f32x4_t *)sk;
#pragma unroll
        for (int e = 0; e < 4; e++) s[e] += v[e];
        if (EPI == EPI_SWIGLU) {
            f32x4_t w = *(const f32x4_t *)(sk + N);
#pragma unroll
            for (int e = 0; e < 4; e++) u[e] += w[e];
        }
    }
    if (EPI == EPI_RESIDUAL) {
        f32x4_t *dst = (f32x4_t *)((float *)C + i);
        f32x4_t v = *dst;
#pragma unroll
        for (int e = 0; e < 4; e++) v[e] += s[e];
        *dst = v;
    } else if (EPI == EPI_SWIGLU) {
        bf16x4_t o;
#pragma unroll
        for (int e = 0; e < 4; e++) o[e] = (bf16_t)vla_silu_mul(s[e], u[e]);
        *(bf16x4_t *)((bf16_t *)C + i) = o;
    } else {
        *(f32x4_t *)((float *)C + i) = s;
    }
}

template <int MB, int EPI>
int launch_mb(const SkinnyParams &p, int n_tiles, hipStream_t st) {
    static bool attr_set = false;
    const size_t lds = 2 * (size_t)MB * 32 * BK * 2;
    if (!attr_set && lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)gemm_skinny_kernel<MB, EPI>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) {
            vla_set_error("hipFuncSetAttribute(gemm_skinny) failed: %s", hipGetErrorString(e));
            return VLA_EHIP;
        }
        attr_set = true;
    }
    dim3 grid(n_tiles, p.splits);
    gemm_skinny_kernel<MB, EPI><<<grid, 256, lds, st>>>(p);
    return vla_check_launch("gemm_skinny");
}

template <int EPI>
int launch_epi(const SkinnyParams &p, int n_tiles, hipStream_t st) {
    if (p.M <= 64) return launch_mb<2, EPI>(p, n_tiles, st);
    if (p.M <= 128) return launch_mb<4, EPI>(p, n_tiles, st);
    return launch_mb<8, EPI>(p, n_tiles, st);
}

}  // namespace

// Adds the split-K partial sums P[splits][M][NP] (NP = N, or 2N for SwiGLU) in split order and applies
// the epilogue.
int launch_splitk_reduce(int epilogue, void *C, const float *P, int splits, int M, int N, hipStream_t st) {
    const int np = (epilogue == EPI_SWIGLU) ? 2 * N : N;
    ProfScope ps("splitk_reduce", (double)(splits + 1) * M * np * 4.0, st);
    size_t MN = (size_t)M * N;
    unsigned blocks = (unsigned)((MN / 4 + 255) / 256);
    if (epilogue == EPI_RESIDUAL) skinny_reduce_kernel<EPI_RESIDUAL><<<blocks, 256, 0, st>>>(C, P, splits, M, N);
    else if (epilogue == EPI_SWIGLU) skinny_reduce_kernel<EPI_SWIGLU><<<blocks, 256, 0, st>>>(C, P, splits, M, N);
    else skinny_reduce_kernel<EPI_STORE><<<blocks, 256, 0, st>>>(C, P, splits, M, N);
    return vla_check_launch("splitk_reduce");
}

static int skinny_target_wgs() { return 512; }      // two workgroups per CU keep the weight stream of 256 CUs busy

size_t gemm_skinny_scratch_bytes(int M, int max_n) {
    return (size_t)8 * M * max_n * sizeof(float);     // at most 8 K-splits of an [M, max_n] fp32 panel
}

// Handles bf16 problems with M <= 256, K a multiple of 64 and segments that are multiples of 128
// weight rows.  `scratch` holds the split-K partials (gemm_skinny_scratch_bytes(M, N), with N
// counting gate and up columns separately).  Returns 1 if handled, 0 if declined.
int try_gemm_bf16_skinny(const GemmArgs &g, void *scratch, hipStream_t st) {
    if (g.kblocked || g.M < 1 || g.M > 256 || g.K % BK != 0 || g.segN % 128 != 0 || !scratch) return 0;
    SkinnyParams p{};
    p.A = (const bf16_t *)g.A;
    p.W0 = (const bf16_t *)g.W[0]; p.W1 = (const bf16_t *)g.W[1]; p.W2 = (const bf16_t *)g.W[2];
    p.C = g.C; p.P = (float *)scratch; p.M = g.M; p.K = g.K; p.segN = g.segN;
    p.N = (g.epilogue == EPI_SWIGLU) ? g.segN : g.n_seg * g.segN;
    const int n_tiles = p.N / 128;
    const int ktiles = g.K / BK;
    // enough workgroups to keep the weight stream of all 256 CUs busy, at least 8 K tiles per split
    int splits = 1;
    while (splits < 8 && n_tiles * splits < skinny_target_wgs() && ktiles / (splits * 2) >= 8) splits *= 2;
    p.splits = splits;
    const double wbytes = 2.0 * g.K * (g.epilogue == EPI_SWIGLU ? 2.0 * p.N : (double)p.N);
    int rc;
    {
        ProfScope ps(g.epilogue == EPI_SWIGLU ? "gemm_skinny<swiglu>" : g.epilogue == EPI_RESIDUAL ? "gemm_skinny<residual>"
                                                                                                   : "gemm_skinny<store>", wbytes, st);
        if (g.epilogue == EPI_SWIGLU) rc = launch_epi<EPI_SWIGLU>(p, n_tiles, st);
        else if (g.epilogue == EPI_RESIDUAL) rc = launch_epi<EPI_RESIDUAL>(p, n_tiles, st);
        else rc = launch_epi<EPI_STORE>(p, n_tiles, st);
        if (rc) return rc;
    }
    if (splits > 1) {
        if (g.deferred_splits && (g.epilogue == EPI_STORE || g.epilogue == EPI_RESIDUAL)) *g.deferred_splits = splits;
        else if ((rc = launch_splitk_reduce(g.epilogue, g.C, p.P, splits, g.M, p.N, st))) return rc;
    }
    return 1;
}
