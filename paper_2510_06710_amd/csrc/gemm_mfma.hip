// bf16 MFMA GEMM for gfx950: C[M, N] = A[M, K] . W[N, K]^T with fp32 accumulation, used for the
// QKV, O, gate/up and down projections of the 7B-shape workloads.
//
// Tiling: a 256-thread workgroup (4 waves, one per SIMD) computes 256 x 256 output tiles and steps K
// by 64 through a double-buffered LDS stage (2 x 64 KB of the CU's 160 KB, so one workgroup per CU).
// Each wave owns a 128 x 128 sub-tile = 4 x 4 blocks of v_mfma_f32_32x32x16_bf16 (256 fp32
// accumulators per lane).  The weight rows are the MFMA's row operand and the activation rows its
// column operand, so a lane ends up with four consecutive output columns of one activation row.
// With more tiles than CUs the grid is one workgroup per CU and each walks its tiles in turn, the
// global loads running two K tiles ahead and straight on into the next tile.
//
// LDS stage: a tile row is 64 bf16 = eight 16-byte chunks; chunk c of row r sits at chunk position
// c ^ ((r >> 1) & 7), which spreads the sixteen rows a quarter-wave reads at once over all banks.
// Global loads are 16 bytes per lane and write LDS linearly (lane t -> 16 * t), the swizzle being
// applied on the global side.
//
// Epilogues (through a per-wave LDS panel, so that memory sees whole rows): store fp32; add into the
// fp32 residual stream; SwiGLU (tile rows interleave 64 gate and 64 up rows per wave so that
// silu(gate) * up pairs two accumulators of the same lane); QKV with the rotation and the KV-cache
// write (q, k, v stay fp32 until after the rotation).  With split K the tile's fp32 partial sums are
// stored instead and reduced by the decode GEMM's reduction kernel.
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

// One accumulator element, moved from its accumulation register to a vector register exactly where the
// epilogue consumes it.  Left to the compiler, all 256 moves are hoisted to the top of the epilogue and
// push the next item's in-flight loads out to scratch memory.
__device__ __forceinline__ float acc_read(const f32x16_t &v, int e) {
    float x;
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x) : "a"(v[e]));
    return x;
}
// The matrix pipe's last results must have landed before the first such move (the assembler text above
// is opaque to the compiler's hazard handling): 2 x 16 idle cycles cover the 16-pass MFMA.
__device__ __forceinline__ void acc_settle() { asm volatile("s_nop 15\n\ts_nop 15"); }

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
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < 4; j++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    f32x4_t v;
#pragma unroll
                    for (int e = 0; e < 4; e++) v[e] = acc_read(acc[j][i], g * 4 + e);
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
        // read-modify-write of the fp32 residual stream through the LDS panel.  x is loaded in whole
        // 512-byte rows, eight 2-row loads per half block, each half issued one block ahead of its use so
        // that the load latency runs under the staging and the stores in between.
        float *out = (float *)p.C + (size_t)tn * BN + wn * 128 + r * 4;
        f32x4_t x[2][8];
        auto load_x = [&](auto half_c, int i) {
            constexpr int HB = decltype(half_c)::value;
            const int mblock = m0 + wm * 128 + i * 32;
#pragma unroll
            for (int it = 0; it < 8; it++) {
                const int m = min(mblock + (HB * 8 + it) * 2 + hh, p.M - 1);
                x[HB][it] = *(const f32x4_t *)(out + (size_t)m * p.N);
            }
        };
        auto add_store = [&](auto half_c, int i) {
            constexpr int HB = decltype(half_c)::value;
            const int mblock = m0 + wm * 128 + i * 32;
#pragma unroll
            for (int it = 0; it < 8; it++) {
                const int row = (HB * 8 + it) * 2 + hh, m = mblock + row;
                f32x4_t v = *(const f32x4_t *)(panel + row * EPI_LD + r * 4);
#pragma unroll
                for (int e = 0; e < 4; e++) v[e] += x[HB][it][e];
                if (m < p.M) *(f32x4_t *)(out + (size_t)m * p.N) = v;
            }
        };
        using H0 = std::integral_constant<int, 0>;
        using H1 = std::integral_constant<int, 1>;
        load_x(H0{}, 0);
        load_x(H1{}, 0);
#pragma unroll
        for (int i = 0; i < 4; i++) {
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < 4; j++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    f32x4_t v;
#pragma unroll
                    for (int e = 0; e < 4; e++) v[e] = acc_read(acc[j][i], g * 4 + e);
                    *(f32x4_t *)(panel + r * EPI_LD + j * 32 + g * 8 + 4 * hh) = v;
                }
            __builtin_amdgcn_sched_barrier(0);
            add_store(H0{}, i);
            if (i < 3) load_x(H0{}, i + 1);
            __builtin_amdgcn_sched_barrier(0);
            add_store(H1{}, i);
            if (i < 3) load_x(H1{}, i + 1);
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const int mblock = m0 + wm * 128 + i * 32;
        // one block at a time: the loads of the next item are in flight in 64 registers across the
        // epilogue, and interleaving all four blocks would push those out to scratch memory
        __builtin_amdgcn_sched_barrier(0);
        // ---- stage ----------------------------------------------------------------------------------
        if (EPI == EPI_SWIGLU) {
#pragma unroll
            for (int j = 0; j < 2; j++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    f32x4_t v;
#pragma unroll
                    for (int e = 0; e < 4; e++) {
                        float gate = acc_read(acc[j][i], g * 4 + e), up = acc_read(acc[j + 2][i], g * 4 + e);
                        v[e] = vla_silu_mul(gate, up);
                    }
                    *(f32x4_t *)(panel + r * EPI_LD + j * 32 + g * 8 + 4 * hh) = v;
                    __builtin_amdgcn_sched_barrier(0);
                }
        } else {
#pragma unroll
            for (int j = 0; j < 4; j++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    f32x4_t v;
#pragma unroll
                    for (int e = 0; e < 4; e++) v[e] = acc_read(acc[j][i], g * 4 + e);
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
                for (int e = 0; e < 4; e++) v[e] = acc_read(acc[j][i], g * 4 + e);
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

// One workgroup walks a list of work items (an output tile, or with SPLITK one K range of a tile)
// `gridDim.x` apart and streams their K tiles through one continuous pipeline: while the last two K
// tiles of an item are multiplied, the first two of the next item are already being fetched, so only
// the very first item of a workgroup pays the load latency of an empty pipeline.
//   SPLITK: items store fp32 partial sums (decode); otherwise the item's epilogue runs here.
// Items with an odd number of K tiles flip the stage parity, so the host launches one workgroup per
// item for those (the loop below then runs once).
template <int EPI, bool SPLITK>
__global__ void __launch_bounds__(256) gemm_bf16_mfma_kernel(MfmaGemmParams p) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    // stage s: A tile at lds + s * 2 * TILE_BYTES, W tile TILE_BYTES after it; the epilogue's panels
    // start at stage 1 and run 2 KB past it
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int n_tiles = p.tiles_m * p.tiles_n;
    const int n_items = n_tiles * p.splits;
    const int K = p.K;
    const int ktiles_all = K / BK;
    int item = blockIdx.x;
    if (item >= n_items) return;

    // ---- load cursor: the K tile the next batch of global loads fetches --------------------------
    // A thread loads chunk (t & 7) of rows i * 32 + (t >> 3), i = 0..7, of both operand tiles; the swizzle
    // depends on the row only through t >> 3, so a single per-thread byte offset serves all sixteen
    // loads.  They are buffer loads: scalar descriptor of the tile's 256 rows + that offset + a scalar
    // offset (K position and row block).  Activation rows past M are read like any other (the caller
    // guarantees the buffer holds whole tiles of rows); their products are never stored.
    const int trow = t >> 3;
    const int thread_off = trow * K * 2 + ((t & 7) ^ swz(trow)) * 16;
    const int tile_bytes = BM * K * 2;
    __amdgpu_buffer_rsrc_t a_rsrc, w_rsrc0, w_rsrc1;
    int ld_item, ld_k, ld_k_end;                     // ld_k in bytes along a row
    int nx_split, nx_tm, nx_tn, nx_nkt;              // the item the cursor is on, for the multiply side
    auto setup_load = [&](int it) {
        const int split = SPLITK ? __builtin_amdgcn_readfirstlane(it / n_tiles) : 0;
        int tm, tn;
        vla_tile_of_block(it - split * n_tiles, p.tiles_m, p.tiles_n, tm, tn);
        a_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)(p.A + (size_t)tm * BM * K), (short)0, tile_bytes, 0x00020000);
        if (EPI == EPI_SWIGLU) {
            w_rsrc0 = __builtin_amdgcn_make_buffer_rsrc((void *)(p.W0 + (size_t)(tn * 128) * K), (short)0, tile_bytes / 2, 0x00020000);
            w_rsrc1 = __builtin_amdgcn_make_buffer_rsrc((void *)(p.W1 + (size_t)(tn * 128) * K), (short)0, tile_bytes / 2, 0x00020000);
        } else {
            const int n = tn * BN;
            const int seg = __builtin_amdgcn_readfirstlane(n / p.segN);
            const bf16_t *Wp = seg == 0 ? p.W0 : (seg == 1 ? p.W1 : p.W2);
            w_rsrc0 = w_rsrc1 = __builtin_amdgcn_make_buffer_rsrc((void *)(Wp + (size_t)(n - seg * p.segN) * K), (short)0, tile_bytes, 0x00020000);
        }
        const int k0 = SPLITK ? (int)((long)split * ktiles_all / p.splits) : 0;
        const int k1 = SPLITK ? (int)((long)(split + 1) * ktiles_all / p.splits) : ktiles_all;
        ld_item = it;
        ld_k = k0 * (BK * 2);
        ld_k_end = k1 * (BK * 2);
        nx_split = split; nx_tm = tm; nx_tn = tn; nx_nkt = k1 - k0;
    };
    // After a batch of loads: next K tile, else the next item's first, else stay on the last tile (it is
    // fetched again and never used: a loop body without a branch around its loads schedules better).
    auto advance = [&]() {
        ld_k += BK * 2;
        if (ld_k == ld_k_end) {
            const int nxt = ld_item + (int)gridDim.x;
            if (nxt < n_items) setup_load(nxt);
            else ld_k -= BK * 2;
        }
    };

    f32x16_t acc[4][4];   // [weight-row block][activation-row block]

    // Two register sets of staged global loads: a tile's loads are issued two K tiles before the tile
    // is multiplied, so a miss that goes past the L2 (all workgroups of an XCD walk K in step and miss
    // on the same lines together) has a full tile time to return.
    bf16x8_t stage_a[2][8], stage_w[2][8];
    auto gload = [&](auto set_c) {
        constexpr int SET = decltype(set_c)::value;
#pragma unroll
        for (int i = 0; i < 8; i++) {
            stage_a[SET][i] = __builtin_bit_cast(bf16x8_t, __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, thread_off, ld_k + i * 32 * K * 2, 0));
            // SwiGLU tiles interleave 64 gate rows and 64 up rows per wave: row blocks g g u u g g u u
            if (EPI == EPI_SWIGLU)
                stage_w[SET][i] = __builtin_bit_cast(bf16x8_t, __builtin_amdgcn_raw_buffer_load_b128(
                    ((i >> 1) & 1) ? w_rsrc1 : w_rsrc0, thread_off, ld_k + ((i >> 2) * 64 + (i & 1) * 32) * K * 2, 0));
            else
                stage_w[SET][i] = __builtin_bit_cast(bf16x8_t, __builtin_amdgcn_raw_buffer_load_b128(w_rsrc0, thread_off, ld_k + i * 32 * K * 2, 0));
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
    // k-step ks+1 are read while the MFMAs of k-step ks run; the global loads of the tile two ahead are
    // issued at the top of a tile, the tile one ahead is written to the other LDS stage during k-step 2,
    // and after one barrier its first fragments are read under the MFMAs of k-step 3.
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

    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    // One K tile; `par` = parity of the tile within the workgroup's stream = its LDS stage = the register
    // set that held it (free again now) and that takes the loads of the tile two ahead.
    auto tile = [&](auto par_c) {
        constexpr int s = decltype(par_c)::value;
        using Other = std::integral_constant<int, s ^ 1>;
        const char *base = lds + s * 2 * TILE_BYTES;
        // Each region below pairs its memory instructions one by one with MFMAs (sched_group_barrier:
        // 0x008 MFMA, 0x020 VMEM read, 0x100 DS read, 0x200 DS write), so the matrix pipe keeps issuing
        // while LDS and global traffic trickles in between.
        gload(par_c);
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
        advance();
    };

    setup_load(item);
    int split = nx_split, tm = nx_tm, tn = nx_tn, nkt = nx_nkt;
    gload(P0{});
    advance();
    gload(P1{});
    advance();
    lstore(P0{}, 0);
    __syncthreads();
    frag_load(0, lds, 0);
    for (; item < n_items; item += (int)gridDim.x) {
#pragma unroll
        for (int j = 0; j < 4; j++)
#pragma unroll
            for (int i = 0; i < 4; i++)
#pragma unroll
                for (int r = 0; r < 16; r++) acc[j][i][r] = 0.f;
        int kt = 0;
        for (; kt + 1 < nkt; kt += 2) {
            tile(P0{});
            tile(P1{});
        }
        if (kt < nkt) tile(P0{});
        // The last barrier of the K loop came after every wave's last read of the stage just multiplied
        // (stage 1 for an even tile count); the other stage already holds the next item's first K tile.
        // The panels go over stage 1; no wave may refill that stage before all panels are drained.
        char *panels = lds + 2 * TILE_BYTES;
        acc_settle();
        if (SPLITK) epilogue_partial<EPI>(acc, p, split, tm * BM, tn, wm, wn, lane, panels);
        else epilogue<EPI>(acc, p, tm * BM, tn, wm, wn, lane, panels);
        __syncthreads();
        // the cursor moved on to the next item (if any) two K tiles before this one ended
        split = nx_split; tm = nx_tm; tn = nx_tn; nkt = nx_nkt;
    }
}

template <int EPI, bool SPLITK>
int launch(const MfmaGemmParams &p, hipStream_t st) {
    static bool attr_set = false;
    static int n_cu = 0;
    const size_t lds = 2 * (size_t)TILE_BYTES + 4 * (size_t)EPI_PANEL_BYTES;      // 130 KB of the CU's 160 KB
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)gemm_bf16_mfma_kernel<EPI, SPLITK>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) {
            vla_set_error("hipFuncSetAttribute(gemm_bf16_mfma) failed: %s", hipGetErrorString(e));
            return VLA_EHIP;
        }
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1) {
            vla_set_error("gemm_bf16_mfma: cannot read the compute-unit count");
            return VLA_EHIP;
        }
        attr_set = true;
    }
    const double flops = 2.0 * p.M * p.K * (EPI == EPI_SWIGLU ? 2.0 * p.N : (double)p.N);
    ProfScope ps(SPLITK ? (EPI == EPI_SWIGLU ? "gemm_bf16_mfma_splitk<swiglu>" : EPI == EPI_RESIDUAL
                           ? "gemm_bf16_mfma_splitk<residual>" : "gemm_bf16_mfma_splitk<store>")
                 : EPI == EPI_SWIGLU ? "gemm_bf16_mfma<swiglu>" : EPI == EPI_RESIDUAL ? "gemm_bf16_mfma<residual>"
                 : EPI == EPI_QKV_ROPE ? "gemm_bf16_mfma<qkv_rope>" : "gemm_bf16_mfma<store>", flops, st);
    // One workgroup fits a CU (130 KB of LDS, 512 registers per lane).  Whole tiles with an even K-tile
    // count are dealt round-robin to one workgroup per CU; blockIdx % 8 is the XCD, and a stride of a
    // multiple of 8 keeps every workgroup's items on its own XCD's share of the tile order.
    int n_items = p.tiles_m * p.tiles_n * p.splits;
    int grid = n_items;
    // (at least four K tiles per item: the load cursor must never be more than one item ahead)
    if (!SPLITK && (p.K / BK) % 2 == 0 && p.K / BK >= 4 && n_cu % 8 == 0 && n_items > n_cu) grid = n_cu;
    gemm_bf16_mfma_kernel<EPI, SPLITK><<<grid, 256, lds, st>>>(p);
    int rc = vla_check_launch("gemm_bf16_mfma");
    return rc ? rc : 1;
}

}  // namespace

// Handles bf16 problems with K a multiple of 64 and N tiles that do not straddle weight segments
// (any M: rows beyond M are loaded from the padded buffer and masked on store, and a row's result does
// not depend on which tile it falls in); anything else is declined (0) and runs on the generic kernel.
int try_gemm_bf16_mfma(const GemmArgs &g, hipStream_t st) {
    if (g.kblocked || g.M < 1 || g.K % BK != 0 || g.a_rows < (g.M + BM - 1) / BM * BM) return 0;
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
    if (g.kblocked || g.M < 1 || g.M > BM || g.a_rows < BM || g.K % BK != 0 || !scratch || g.epilogue == EPI_QKV_ROPE) return 0;
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
