// bf16 MFMA GEMM for gfx950: C[M, N] = A[M, K] . W[N, K]^T with fp32 accumulation, used for the
// QKV, O, gate/up and down projections of the 7B-shape workloads.
//
// Tiling: one 256-thread workgroup (4 waves, one per SIMD) owns a 256 x 256 output tile and steps K
// by 64 through a double-buffered LDS stage (2 x 64 KB of the CU's 160 KB).  Each wave owns a
// 128 x 128 sub-tile = 4 x 4 blocks of v_mfma_f32_32x32x16_bf16 (256 fp32 accumulators per lane).
// The weight rows are the MFMA's row operand and the activation rows its column operand, so a lane
// ends up with four consecutive output columns of one activation row: 8-byte bf16 / 16-byte fp32
// stores in the epilogue.
//
// LDS stage: a tile row is 64 bf16 = eight 16-byte chunks; chunk c of row r sits at chunk position
// c ^ ((r >> 1) & 7), which spreads the sixteen rows a quarter-wave reads at once over all banks.
// Global loads are 16 bytes per lane and write LDS linearly (lane t -> 16 * t), the swizzle being
// applied on the global side.
//
// Epilogues: store fp32 (QKV, rounded only after the rotation); add into the fp32 residual stream; SwiGLU (tile rows interleave 64 gate and
// 64 up rows per wave so that silu(gate) * up pairs two accumulators of the same lane).
#include <stdlib.h>

#include "vla_internal.h"

namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int TILE_BYTES = BM * BK * 2;     // 32 KB per operand per stage

struct MfmaGemmParams {
    const bf16_t *A;
    const bf16_t *W0, *W1, *W2;
    void *C;
    int M, N, K, segN;
    int tiles_m, tiles_n;
    int dbg;
};

__device__ __forceinline__ int swz(int row) { return (row >> 1) & 7; }

// Maps the linear workgroup id to an output tile.  Workgroups are dealt round-robin to the eight
// XCDs, each with its own L2: ids of one XCD are made contiguous, then walked in column panels
// of `GROUP` tile rows so that the ~32 tiles resident on an XCD share activation and weight rows.
__device__ __forceinline__ void tile_of_block(int pid, int tiles_m, int tiles_n, int &tm, int &tn) {
    int total = tiles_m * tiles_n;
    int per_xcd = (total + 7) / 8;
    int xcd = pid % 8, local = pid / 8;
    int lin = xcd * per_xcd + local;
    if (per_xcd * 8 != total) lin = pid;     // ragged tile counts: keep the plain order
    constexpr int GROUP = 8;
    int panel = lin / (GROUP * tiles_n);
    int first_m = panel * GROUP;
    int rows = min(GROUP, tiles_m - first_m);
    int in_panel = lin - panel * GROUP * tiles_n;
    tm = first_m + in_panel % rows;
    tn = in_panel / rows;
}

template <int EPI>
__global__ void __launch_bounds__(256) gemm_bf16_mfma_kernel(MfmaGemmParams p) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    // stage s: A tile at lds + s * 2 * TILE_BYTES, W tile TILE_BYTES after it
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    int tm, tn;
    tile_of_block(blockIdx.x, p.tiles_m, p.tiles_n, tm, tn);
    const int m0 = tm * BM;
    const int K = p.K;

    // ---- per-thread global sources: 8 chunks of A and 8 chunks of W per K tile -----------------
    const bf16_t *asrc[8], *wsrc[8];
#pragma unroll
    for (int i = 0; i < 8; i++) {
        int q = i * 256 + t;
        int row = q >> 3, pc = q & 7;
        int c = pc ^ swz(row);
        int m = min(m0 + row, p.M - 1);
        asrc[i] = p.A + (size_t)m * K + c * 8;
        const bf16_t *wrow;
        if (EPI == EPI_SWIGLU) {
            int sub = row >> 6;
            int f = tn * 128 + (sub >> 1) * 64 + (row & 63);
            wrow = ((sub & 1) ? p.W1 : p.W0) + (size_t)f * K;
        } else {
            int n = tn * BN + row;
            int seg = n / p.segN;
            const bf16_t *Wp = seg == 0 ? p.W0 : (seg == 1 ? p.W1 : p.W2);
            wrow = Wp + (size_t)(n - seg * p.segN) * K;
        }
        wsrc[i] = wrow + c * 8;
    }

    f32x16_t acc[4][4];   // [weight-row block][activation-row block]
#pragma unroll
    for (int j = 0; j < 4; j++)
#pragma unroll
        for (int i = 0; i < 4; i++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[j][i][r] = 0.f;

    bf16x8_t stage_a[8], stage_w[8];
    auto gload = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 8; i++) {
            stage_a[i] = *(const bf16x8_t *)(asrc[i] + k0);
            stage_w[i] = *(const bf16x8_t *)(wsrc[i] + k0);
        }
    };
    auto lstore = [&](int s) {
        char *base = lds + s * 2 * TILE_BYTES;
#pragma unroll
        for (int i = 0; i < 8; i++) {
            *(bf16x8_t *)(base + (i * 256 + t) * 16) = stage_a[i];
            *(bf16x8_t *)(base + TILE_BYTES + (i * 256 + t) * 16) = stage_w[i];
        }
    };

    // fragment addresses inside a tile: row * 128 + ((kstep * 2 + lane / 32) ^ swz(row)) * 16
    int a_off[4], w_off[4], a_sw[4], w_sw[4];
#pragma unroll
    for (int i = 0; i < 4; i++) {
        int ra = wm * 128 + i * 32 + (lane & 31);
        int rw = wn * 128 + i * 32 + (lane & 31);
        a_off[i] = ra * 128; a_sw[i] = swz(ra);
        w_off[i] = TILE_BYTES + rw * 128; w_sw[i] = swz(rw);
    }
    const int khalf = lane >> 5;

    // Software pipeline (one wave per SIMD, so nothing else hides LDS latency): the fragments of
    // k-step ks+1 are read while the MFMAs of k-step ks run; the next K tile's global loads are issued
    // at the top of the tile, written to the other LDS stage during k-step 2, and after one barrier
    // the first fragments of the next tile are read under the MFMAs of k-step 3.
    bf16x8_t af[2][4], wf[2][4];
    auto frag_load = [&](int buf, const char *base, int ks) {
        const int c = ks * 2 + khalf;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            af[buf][i] = *(const bf16x8_t *)(base + a_off[i] + ((c ^ a_sw[i]) << 4));
            wf[buf][i] = *(const bf16x8_t *)(base + w_off[i] + ((c ^ w_sw[i]) << 4));
        }
    };
    auto mfma_step = [&](int buf) {
#pragma unroll
        for (int j = 0; j < 4; j++)
#pragma unroll
            for (int i = 0; i < 4; i++)
                acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[buf][j], af[buf][i], acc[j][i], 0, 0, 0);
    };

    const int ktiles = K / BK;
    gload(0);
    lstore(0);
    __syncthreads();
    frag_load(0, lds, 0);
    for (int kt = 0; kt < ktiles; kt++) {
        const int s = kt & 1;
        // the last tile re-stages itself into the idle buffer: a branch-free body schedules better
        const int kn = p.dbg ? 0 : min(kt + 1, ktiles - 1);
        const char *base = lds + s * 2 * TILE_BYTES;
        // Each region below pairs its memory instructions one by one with MFMAs (sched_group_barrier:
        // 0x008 MFMA, 0x020 VMEM read, 0x100 DS read, 0x200 DS write), so the matrix pipe keeps issuing
        // while LDS and global traffic trickles in between.
        gload(kn * BK);
        frag_load(1, base, 1);
        mfma_step(0);
#pragma unroll
        for (int i = 0; i < 8; i++) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
#pragma unroll
        for (int i = 0; i < 8; i++) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        frag_load(0, base, 2);
        mfma_step(1);
#pragma unroll
        for (int i = 0; i < 8; i++) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
        __builtin_amdgcn_sched_barrier(0);
        frag_load(1, base, 3);
        lstore(s ^ 1);
        mfma_step(0);
#pragma unroll
        for (int i = 0; i < 8; i++) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
#pragma unroll
        for (int i = 0; i < 8; i++) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x200, 2, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        frag_load(0, lds + (s ^ 1) * 2 * TILE_BYTES, 0);
        mfma_step(1);
#pragma unroll
        for (int i = 0; i < 8; i++) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
        __builtin_amdgcn_sched_barrier(0);
    }

    // ---- epilogue: lane holds activation row m = .. + lane % 32 and, per accumulator register r,
    // weight row 8 * (r / 4) + 4 * (lane / 32) + r % 4 of its block --------------------------------
    const int mrow_base = m0 + wm * 128 + (lane & 31);
    const int nquad = 4 * (lane >> 5);
#pragma unroll
    for (int i = 0; i < 4; i++) {
        int m = mrow_base + i * 32;
        if (m >= p.M) continue;
        if (EPI == EPI_SWIGLU) {
            bf16_t *out = (bf16_t *)p.C + (size_t)m * p.N + tn * 128 + wn * 64;
#pragma unroll
            for (int j = 0; j < 2; j++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    bf16x4_t o;
#pragma unroll
                    for (int e = 0; e < 4; e++) {
                        float gate = acc[j][i][g * 4 + e], up = acc[j + 2][i][g * 4 + e];
                        o[e] = (bf16_t)(gate / (1.0f + __expf(-gate)) * up);
                    }
                    *(bf16x4_t *)(out + j * 32 + g * 8 + nquad) = o;
                }
        } else if (EPI == EPI_RESIDUAL) {
            float *out = (float *)p.C + (size_t)m * p.N + tn * BN + wn * 128;
#pragma unroll
            for (int j = 0; j < 4; j++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    f32x4_t *dst = (f32x4_t *)(out + j * 32 + g * 8 + nquad);
                    f32x4_t v = *dst;
#pragma unroll
                    for (int e = 0; e < 4; e++) v[e] += acc[j][i][g * 4 + e];
                    *dst = v;
                }
        } else {
            float *out = (float *)p.C + (size_t)m * p.N + tn * BN + wn * 128;
#pragma unroll
            for (int j = 0; j < 4; j++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    f32x4_t v;
#pragma unroll
                    for (int e = 0; e < 4; e++) v[e] = acc[j][i][g * 4 + e];
                    *(f32x4_t *)(out + j * 32 + g * 8 + nquad) = v;
                }
        }
    }
}

template <int EPI>
int launch(const MfmaGemmParams &p, hipStream_t st) {
    static bool attr_set = false;
    const size_t lds = 4 * (size_t)TILE_BYTES;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)gemm_bf16_mfma_kernel<EPI>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) {
            vla_set_error("hipFuncSetAttribute(gemm_bf16_mfma) failed: %s", hipGetErrorString(e));
            return VLA_EHIP;
        }
        attr_set = true;
    }
    const double flops = 2.0 * p.M * p.K * (EPI == EPI_SWIGLU ? 2.0 * p.N : (double)p.N);
    ProfScope ps(EPI == EPI_SWIGLU ? "gemm_bf16_mfma<swiglu>" : EPI == EPI_RESIDUAL ? "gemm_bf16_mfma<residual>"
                                                                                 : "gemm_bf16_mfma<store>", flops, st);
    gemm_bf16_mfma_kernel<EPI><<<p.tiles_m * p.tiles_n, 256, lds, st>>>(p);
    int rc = vla_check_launch("gemm_bf16_mfma");
    return rc ? rc : 1;
}

}  // namespace

// Handles bf16 problems with K a multiple of 64 and N tiles that do not straddle weight segments
// (any M: rows beyond M are clamped on load and masked on store, and a row's result does not
// depend on which tile it falls in); anything else is declined (0) and runs on the generic kernel.
int try_gemm_bf16_mfma(const GemmArgs &g, hipStream_t st) {
    if (g.M < 1 || g.K % BK != 0) return 0;
    MfmaGemmParams p{};
    p.A = (const bf16_t *)g.A;
    p.W0 = (const bf16_t *)g.W[0]; p.W1 = (const bf16_t *)g.W[1]; p.W2 = (const bf16_t *)g.W[2];
    p.C = g.C; p.M = g.M; p.K = g.K; p.segN = g.segN;
    p.tiles_m = (g.M + BM - 1) / BM;
    { const char *e = getenv("VLA_GEMM_DBG"); p.dbg = e ? atoi(e) : 0; }
    if (g.epilogue == EPI_SWIGLU) {
        if (g.segN % 128 != 0) return 0;
        p.N = g.segN;
        p.tiles_n = g.segN / 128;
        return launch<EPI_SWIGLU>(p, st);
    }
    if (g.segN % BN != 0) return 0;
    p.N = g.n_seg * g.segN;
    p.tiles_n = p.N / BN;
    return g.epilogue == EPI_RESIDUAL ? launch<EPI_RESIDUAL>(p, st) : launch<EPI_STORE>(p, st);
}
