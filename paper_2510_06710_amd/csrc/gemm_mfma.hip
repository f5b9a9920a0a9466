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
#include "vla_internal.h"

#include <type_traits>

namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int TILE_BYTES = BM * BK * 2;     // 32 KB per operand per stage

struct MfmaGemmParams {
    const bf16_t *A;
    const bf16_t *W0, *W1, *W2;
    void *C;
    int M, N, K, segN;
    int tiles_m, tiles_n;
    int splits;      // K split across workgroups (decode at M > 128); partial sums go to P
    float *P;        // [splits][M][N] fp32 (SwiGLU: [splits][M][2N], gate columns then up columns)
    // EPI_QKV_ROPE
    bf16_t *q_out, *kc, *vc;
    const float2 *table;
    int R, pos0, n_heads, pos_stride, H;
};

__device__ __forceinline__ int swz(int row) { return (row >> 1) & 7; }

// Maps the linear workgroup id to an output tile.  Workgroups are dealt round-robin to the eight
// XCDs, each with its own L2: ids of one XCD are made contiguous, then walked in column panels
// of `GROUP` tile rows so that the ~32 tiles resident on an XCD (4 x 8) share activation and weight rows.
__device__ __forceinline__ void tile_of_block(int pid, int tiles_m, int tiles_n, int &tm, int &tn) {
    int total = tiles_m * tiles_n;
    int per_xcd = (total + 7) / 8;
    int xcd = pid % 8, local = pid / 8;
    int lin = xcd * per_xcd + local;
    if (per_xcd * 8 != total) lin = pid;     // ragged tile counts: keep the plain order
    constexpr int GROUP = 4;                 // measured best of 1, 2, 4, 6, 8, 16, 32 on the 7B shapes
    int panel = lin / (GROUP * tiles_n);
    int first_m = panel * GROUP;
    int rows = min(GROUP, tiles_m - first_m);
    int in_panel = lin - panel * GROUP * tiles_n;
    tm = first_m + in_panel % rows;
    tn = in_panel / rows;
}

// Output of one wave.  A lane holds activation row (lane % 32) of each 32-row block and, per
// accumulator register r, weight row 8 * (r / 4) + 4 * (lane / 32) + r % 4: written out directly that is
// 32-byte pieces of 32 different rows per store instruction.  Instead each 32 x 128 block goes through
// a per-wave LDS panel (row stride 132 floats: the 16 lanes of a quarter-wave hit all 64 banks) and
// leaves as whole rows: a store (or the load + store of the residual update) covers two 512-byte rows,
// the bf16 SwiGLU output eight 128-byte rows.
constexpr int EPI_LD = 132;                               // floats per staged row
constexpr int EPI_PANEL_BYTES = 32 * EPI_LD * 4;          // 16.5 KB per wave

template <int EPI>
__device__ __forceinline__ void epilogue(f32x16_t (&acc)[4][4], const MfmaGemmParams &p, int m0, int tn, int wm,
                                         int wn, int lane, char *lds_all) {
    float *panel = (float *)(lds_all + (wm * 2 + wn) * EPI_PANEL_BYTES);
    const int r = lane & 31, hh = lane >> 5;
    if (EPI == EPI_QKV_ROPE) {
        // The wave's 128 columns are one head of q, k or v (head_dim 128).  Each 32-row block is staged
        // in the LDS panel, then q and k are rotated (pairs (i, i + 64), angles from the table) and
        // written as bf16: q to its [M, H] buffer, k to the [d/8][position][8] layout with the 32 lanes
        // of a half-wave on 32 consecutive positions of one chunk, v to [position][d].
        const int n0 = tn * BN + wn * 128;
        const int seg = n0 / p.H, head = (n0 - seg * p.H) >> 7;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int mblock = m0 + wm * 128 + i * 32;
#pragma unroll
            for (int j = 0; j < 4; j++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    f32x4_t v;
#pragma unroll
                    for (int e = 0; e < 4; e++) v[e] = acc[j][i][g * 4 + e];
                    *(f32x4_t *)(panel + r * EPI_LD + j * 32 + g * 8 + 4 * hh) = v;
                }
            if (seg == 2) {
#pragma unroll
                for (int it = 0; it < 8; it++) {
                    const int row = it * 4 + (lane >> 4), c = lane & 15, m = mblock + row;
                    f32x4_t a = *(const f32x4_t *)(panel + row * EPI_LD + c * 8);
                    f32x4_t b = *(const f32x4_t *)(panel + row * EPI_LD + c * 8 + 4);
                    bf16x8_t o;
#pragma unroll
                    for (int e = 0; e < 4; e++) { o[e] = (bf16_t)a[e]; o[4 + e] = (bf16_t)b[e]; }
                    if (m < p.M) {
                        const int sq = m / p.R, pos = p.pos0 + (m - sq * p.R);
                        *(bf16x8_t *)(p.vc + (((size_t)sq * p.n_heads + head) * p.pos_stride + pos) * 128 + c * 8) = o;
                    }
                }
            } else {
#pragma unroll
                for (int it = 0; it < 4; it++) {
                    // q: consecutive lanes take consecutive chunks of a row; k: consecutive positions of a chunk
                    const int item = it * 64 + lane;
                    const int row = (seg == 0) ? (item >> 3) : (item & 31);
                    const int c = (seg == 0) ? (item & 7) : (item >> 5);
                    const int m = mblock + row;
                    const float *src = panel + row * EPI_LD + c * 8;
                    f32x4_t lo0 = *(const f32x4_t *)src, lo1 = *(const f32x4_t *)(src + 4);
                    f32x4_t hi0 = *(const f32x4_t *)(src + 64), hi1 = *(const f32x4_t *)(src + 68);
                    if (m < p.M) {
                        const int sq = m / p.R, rr = m - sq * p.R, pos = p.pos0 + rr;
                        const f32x4_t *tb = (const f32x4_t *)(p.table + (size_t)rr * 64 + c * 8);
                        bf16x8_t olo, ohi;
#pragma unroll
                        for (int e2 = 0; e2 < 4; e2++) {
                            const f32x4_t cs = tb[e2];        // (cos, sin) of dims 2 e2 and 2 e2 + 1 of the chunk
#pragma unroll
                            for (int u = 0; u < 2; u++) {
                                const int e = 2 * e2 + u;
                                const float co = cs[2 * u], si = cs[2 * u + 1];
                                const float a = e < 4 ? lo0[e & 3] : lo1[e & 3], b = e < 4 ? hi0[e & 3] : hi1[e & 3];
                                olo[e] = (bf16_t)(a * co - b * si);
                                ohi[e] = (bf16_t)(b * co + a * si);
                            }
                        }
                        if (seg == 0) {
                            bf16_t *q = p.q_out + (size_t)m * p.H + head * 128 + c * 8;
                            *(bf16x8_t *)q = olo;
                            *(bf16x8_t *)(q + 64) = ohi;
                        } else {
                            const size_t hb = ((size_t)sq * p.n_heads + head) * 16;
                            *(bf16x8_t *)(p.kc + ((hb + c) * p.pos_stride + pos) * 8) = olo;
                            *(bf16x8_t *)(p.kc + ((hb + 8 + c) * p.pos_stride + pos) * 8) = ohi;
                        }
                    }
                }
            }
        }
        return;
    }
    if (EPI == EPI_RESIDUAL) {
        // read-modify-write of the fp32 residual stream through the LDS panel: per 32-row block all
        // sixteen 2-row loads of x are issued first (whole 512-byte rows), then added and stored
        float *out = (float *)p.C + (size_t)tn * BN + wn * 128 + r * 4;
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int mblock = m0 + wm * 128 + i * 32;
            f32x4_t x[16];
#pragma unroll
            for (int it = 0; it < 16; it++) {
                const int m = min(mblock + it * 2 + hh, p.M - 1);
                x[it] = *(const f32x4_t *)(out + (size_t)m * p.N);
            }
#pragma unroll
            for (int j = 0; j < 4; j++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    f32x4_t v;
#pragma unroll
                    for (int e = 0; e < 4; e++) v[e] = acc[j][i][g * 4 + e];
                    *(f32x4_t *)(panel + r * EPI_LD + j * 32 + g * 8 + 4 * hh) = v;
                }
#pragma unroll
            for (int it = 0; it < 16; it++) {
                const int row = it * 2 + hh, m = mblock + row;
                f32x4_t v = *(const f32x4_t *)(panel + row * EPI_LD + r * 4);
#pragma unroll
                for (int e = 0; e < 4; e++) v[e] += x[it][e];
                if (m < p.M) *(f32x4_t *)(out + (size_t)m * p.N) = v;
            }
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const int mblock = m0 + wm * 128 + i * 32;
        // ---- stage ----------------------------------------------------------------------------------
        if (EPI == EPI_SWIGLU) {
#pragma unroll
            for (int j = 0; j < 2; j++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    f32x4_t v;
#pragma unroll
                    for (int e = 0; e < 4; e++) {
                        float gate = acc[j][i][g * 4 + e], up = acc[j + 2][i][g * 4 + e];
                        v[e] = gate / (1.0f + __expf(-gate)) * up;
                    }
                    *(f32x4_t *)(panel + r * EPI_LD + j * 32 + g * 8 + 4 * hh) = v;
                }
        } else {
#pragma unroll
            for (int j = 0; j < 4; j++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    f32x4_t v;
#pragma unroll
                    for (int e = 0; e < 4; e++) v[e] = acc[j][i][g * 4 + e];
                    *(f32x4_t *)(panel + r * EPI_LD + j * 32 + g * 8 + 4 * hh) = v;
                }
        }
        // ---- write out whole rows -------------------------------------------------------------------
        if (EPI == EPI_SWIGLU) {
            bf16_t *out = (bf16_t *)p.C + (size_t)tn * 128 + wn * 64 + (lane & 7) * 8;
#pragma unroll
            for (int it = 0; it < 4; it++) {
                const int row = it * 8 + (lane >> 3), m = mblock + row;
                f32x4_t a = *(const f32x4_t *)(panel + row * EPI_LD + (lane & 7) * 8);
                f32x4_t b = *(const f32x4_t *)(panel + row * EPI_LD + (lane & 7) * 8 + 4);
                bf16x8_t o;
#pragma unroll
                for (int e = 0; e < 4; e++) { o[e] = (bf16_t)a[e]; o[4 + e] = (bf16_t)b[e]; }
                if (m < p.M) *(bf16x8_t *)(out + (size_t)m * p.N) = o;
            }
        } else {
            float *out = (float *)p.C + (size_t)tn * BN + wn * 128 + r * 4;
#pragma unroll
            for (int it = 0; it < 16; it++) {
                const int row = it * 2 + hh, m = mblock + row;
                f32x4_t v = *(const f32x4_t *)(panel + row * EPI_LD + r * 4);
                if (m < p.M) *(f32x4_t *)(out + (size_t)m * p.N) = v;
            }
        }
    }
}

// Split-K: the wave's 32 x 128 blocks leave as fp32 partial sums, whole rows at a time, for the ordered
// reduction kernel.  SwiGLU tiles carry 64 gate and 64 up columns per wave: gate goes to column f, up to
// column N + f of a [M][2N] panel.
template <int EPI>
__device__ __forceinline__ void epilogue_partial(f32x16_t (&acc)[4][4], const MfmaGemmParams &p, int split, int m0,
                                                 int tn, int wm, int wn, int lane, char *lds_all) {
    float *panel = (float *)(lds_all + (wm * 2 + wn) * EPI_PANEL_BYTES);
    const int r = lane & 31, hh = lane >> 5;
    const int NP = (EPI == EPI_SWIGLU) ? 2 * p.N : p.N;
    int col;
    if (EPI == EPI_SWIGLU) col = (r < 16 ? 0 : p.N - 64) + tn * 128 + wn * 64 + r * 4;   // r >= 16: up half
    else col = tn * BN + wn * 128 + r * 4;
    float *out = p.P + (size_t)split * p.M * NP + col;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const int mblock = m0 + wm * 128 + i * 32;
#pragma unroll
        for (int j = 0; j < 4; j++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
                f32x4_t v;
#pragma unroll
                for (int e = 0; e < 4; e++) v[e] = acc[j][i][g * 4 + e];
                *(f32x4_t *)(panel + r * EPI_LD + j * 32 + g * 8 + 4 * hh) = v;
            }
#pragma unroll
        for (int it = 0; it < 16; it++) {
            const int row = it * 2 + hh, m = mblock + row;
            f32x4_t v = *(const f32x4_t *)(panel + row * EPI_LD + r * 4);
            if (m < p.M) *(f32x4_t *)(out + (size_t)m * NP) = v;
        }
    }
}

// SPLITK: each workgroup takes one K range of one tile and stores fp32 partial sums (decode);
// otherwise a workgroup owns a whole tile and runs the epilogue itself (prefill, recompute).
template <int EPI, bool SPLITK>
__global__ void __launch_bounds__(256) gemm_bf16_mfma_kernel(MfmaGemmParams p) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    // stage s: A tile at lds + s * 2 * TILE_BYTES, W tile TILE_BYTES after it
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    int tm, tn;
    const int n_tiles = p.tiles_m * p.tiles_n;
    const int split = SPLITK ? blockIdx.x / n_tiles : 0;
    tile_of_block(blockIdx.x - split * n_tiles, p.tiles_m, p.tiles_n, tm, tn);
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

    // Two register sets of staged global loads: a tile's loads are issued two K tiles before the tile
    // is multiplied, so a miss that goes past the L2 (all workgroups of an XCD walk K in step and miss
    // on the same lines together) has a full tile time to return.
    bf16x8_t stage_a[2][8], stage_w[2][8];
    auto gload = [&](auto set_c, int k0) {
        constexpr int SET = decltype(set_c)::value;
#pragma unroll
        for (int i = 0; i < 8; i++) {
            stage_a[SET][i] = *(const bf16x8_t *)(asrc[i] + k0);
            stage_w[SET][i] = *(const bf16x8_t *)(wsrc[i] + k0);
        }
    };
    auto lstore = [&](auto set_c, int s) {
        constexpr int SET = decltype(set_c)::value;
        char *base = lds + s * 2 * TILE_BYTES;
#pragma unroll
        for (int i = 0; i < 8; i++) {
            *(bf16x8_t *)(base + (i * 256 + t) * 16) = stage_a[SET][i];
            *(bf16x8_t *)(base + TILE_BYTES + (i * 256 + t) * 16) = stage_w[SET][i];
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

    const int ktiles_all = K / BK;
    const int kt0 = SPLITK ? (int)((long)split * ktiles_all / p.splits) : 0;
    const int ktiles = SPLITK ? (int)((long)(split + 1) * ktiles_all / p.splits) : ktiles_all;
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    gload(P0{}, kt0 * BK);
    gload(P1{}, min(kt0 + 1, ktiles - 1) * BK);
    lstore(P0{}, 0);
    __syncthreads();
    frag_load(0, lds, 0);
    // One K tile; `par` = parity of the tile within this workgroup's K range = its LDS stage = the
    // register set that held it (free again now) and that takes the loads of the tile two ahead.
    auto tile = [&](auto par_c, int kt) {
        constexpr int s = decltype(par_c)::value;
        using Other = std::integral_constant<int, s ^ 1>;
        // the last tiles re-stage the final tile: a branch-free body schedules better
        const int kn = min(kt + 2, ktiles - 1);
        const char *base = lds + s * 2 * TILE_BYTES;
        // Each region below pairs its memory instructions one by one with MFMAs (sched_group_barrier:
        // 0x008 MFMA, 0x020 VMEM read, 0x100 DS read, 0x200 DS write), so the matrix pipe keeps issuing
        // while LDS and global traffic trickles in between.
        gload(par_c, kn * BK);
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
        lstore(Other{}, s ^ 1);
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
    };
    int kt = kt0;
    for (; kt + 1 < ktiles; kt += 2) {
        tile(P0{}, kt);
        tile(P1{}, kt + 1);
    }
    if (kt < ktiles) tile(P0{}, kt);

    __syncthreads();                          // every wave is done reading operand tiles: LDS is reused
    if (SPLITK) epilogue_partial<EPI>(acc, p, split, m0, tn, wm, wn, lane, lds);
    else epilogue<EPI>(acc, p, m0, tn, wm, wn, lane, lds);
}

template <int EPI, bool SPLITK>
int launch(const MfmaGemmParams &p, hipStream_t st) {
    static bool attr_set = false;
    const size_t lds = 4 * (size_t)TILE_BYTES;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)gemm_bf16_mfma_kernel<EPI, SPLITK>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) {
            vla_set_error("hipFuncSetAttribute(gemm_bf16_mfma) failed: %s", hipGetErrorString(e));
            return VLA_EHIP;
        }
        attr_set = true;
    }
    const double flops = 2.0 * p.M * p.K * (EPI == EPI_SWIGLU ? 2.0 * p.N : (double)p.N);
    ProfScope ps(SPLITK ? (EPI == EPI_SWIGLU ? "gemm_bf16_mfma_splitk<swiglu>" : EPI == EPI_RESIDUAL
                           ? "gemm_bf16_mfma_splitk<residual>" : "gemm_bf16_mfma_splitk<store>")
                 : EPI == EPI_SWIGLU ? "gemm_bf16_mfma<swiglu>" : EPI == EPI_RESIDUAL ? "gemm_bf16_mfma<residual>"
                 : EPI == EPI_QKV_ROPE ? "gemm_bf16_mfma<qkv_rope>" : "gemm_bf16_mfma<store>", flops, st);
    gemm_bf16_mfma_kernel<EPI, SPLITK><<<p.tiles_m * p.tiles_n * p.splits, 256, lds, st>>>(p);
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
    p.splits = 1;
    if (g.epilogue == EPI_SWIGLU) {
        if (g.segN % 128 != 0) return 0;
        p.N = g.segN;
        p.tiles_n = g.segN / 128;
        return launch<EPI_SWIGLU, false>(p, st);
    }
    if (g.segN % BN != 0) return 0;
    if (g.epilogue == EPI_QKV_ROPE) {
        const QkvRopeArgs *ra = g.rope;
        if (!ra || ra->kv->d != 128 || g.n_seg != 3 || g.segN != ra->kv->n_heads * 128) return 0;
        p.q_out = (bf16_t *)ra->q_out;
        p.kc = (bf16_t *)ra->kv->k + (size_t)ra->layer * ra->kv->layer_elems;
        p.vc = (bf16_t *)ra->kv->v + (size_t)ra->layer * ra->kv->layer_elems;
        p.table = ra->table;
        p.R = ra->rows->R; p.pos0 = ra->rows->pos0; p.n_heads = ra->kv->n_heads;
        p.pos_stride = ra->kv->pos_stride; p.H = g.segN;
        p.N = 3 * g.segN;
        p.tiles_n = p.N / BN;
        return launch<EPI_QKV_ROPE, false>(p, st);
    }
    p.N = g.n_seg * g.segN;
    p.tiles_n = p.N / BN;
    return g.epilogue == EPI_RESIDUAL ? launch<EPI_RESIDUAL, false>(p, st) : launch<EPI_STORE, false>(p, st);
}

// Decode forwards with more than 128 rows: the large tile with K split over workgroups so that the
// single row of tiles still covers the chip; partial sums are reduced in split order by the decode
// GEMM's reduction kernel (no atomics).  `scratch` holds the partials.
int try_gemm_bf16_mfma_splitk(const GemmArgs &g, void *scratch, size_t scratch_bytes, hipStream_t st) {
    if (g.M < 1 || g.M > BM || g.K % BK != 0 || !scratch || g.epilogue == EPI_QKV_ROPE) return 0;
    MfmaGemmParams p{};
    p.A = (const bf16_t *)g.A;
    p.W0 = (const bf16_t *)g.W[0]; p.W1 = (const bf16_t *)g.W[1]; p.W2 = (const bf16_t *)g.W[2];
    p.C = g.C; p.M = g.M; p.K = g.K; p.segN = g.segN;
    p.tiles_m = 1;
    int np;
    if (g.epilogue == EPI_SWIGLU) {
        if (g.segN % 128 != 0) return 0;
        p.N = g.segN; p.tiles_n = g.segN / 128; np = 2 * p.N;
    } else {
        if (g.segN % BN != 0) return 0;
        p.N = g.n_seg * g.segN; p.tiles_n = p.N / BN; np = p.N;
    }
    const int ktiles = g.K / BK;
    int splits = (256 + p.tiles_n / 2) / p.tiles_n;          // about one workgroup per CU
    if (splits > ktiles / 4) splits = ktiles / 4;              // at least four K tiles per split
    if (splits > 16) splits = 16;
    while (splits > 1 && (size_t)splits * g.M * np * sizeof(float) > scratch_bytes) splits--;
    if (splits < 1) splits = 1;
    p.splits = splits;
    p.P = (float *)scratch;
    int rc;
    if (splits == 1) {                                         // no room for partials: whole tiles
        if (g.epilogue == EPI_SWIGLU) return launch<EPI_SWIGLU, false>(p, st);
        return g.epilogue == EPI_RESIDUAL ? launch<EPI_RESIDUAL, false>(p, st) : launch<EPI_STORE, false>(p, st);
    }
    if (g.epilogue == EPI_SWIGLU) rc = launch<EPI_SWIGLU, true>(p, st);
    else if (g.epilogue == EPI_RESIDUAL) rc = launch<EPI_RESIDUAL, true>(p, st);
    else rc = launch<EPI_STORE, true>(p, st);
    if (rc < 0) return rc;
    if ((rc = launch_splitk_reduce(g.epilogue, g.C, p.P, splits, g.M, p.N, st))) return rc;
    return 1;
}
