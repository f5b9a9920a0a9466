// bf16 MFMA GEMM for gfx950 with direct-to-LDS loads: C[M, N] = A[M, K] . W[N, K]^T, fp32 accumulation.
// This is the kernel of the prefill / recompute / parallel-chunk projections (whole tiles), and, with K cut into
// equal ranges whose fp32 partial products go to a scratch buffer, of the QKV and gate/up projections of decode
// forwards of 129..256 rows.
//
// Tiling: 256 x 256 output tiles, 4 waves (one per SIMD), 128 x 128 per wave as 8 x 8 blocks of
// v_mfma_f32_16x16x32_bf16 (256 fp32 accumulators per lane).  The weight rows are the MFMA's row
// operand and the activation rows its column operand: a lane ends up with activation row (lane % 16) of
// a block and four consecutive output columns.
//
// K moves in half tiles of 32 through a ring of four 32 KB LDS stages.  `buffer_load ... lds` writes
// the operands straight into LDS (no staging registers, no ds_write): a wave instruction fills 1 KB
// linearly, i.e. 16 tile rows of 64 bytes; chunk c (16 bytes) of row r sits at position
// c ^ ((r >> 1) & 3), chosen on the global side by which chunk a lane fetches, so that the fragment
// reads are free of bank conflicts: a ds_read_b128 is served eight lanes (128 bytes) at a time, and the eight
// 64-byte rows of such a group then cover the eight 16-byte slots of 128 bytes (with (r >> 2) & 3, which would
// suit 256 bytes per step, SQ_LDS_BANK_CONFLICT showed every read taking twice as long).  The loads of half tile g + 3 are issued while half tile g is read.
//
// Schedule of one iteration g (one barrier): wait for this wave's loads of half tile g, barrier, then 16
// groups of {one ds_read_b128 of half tile g into fragment buffer g % 2, four MFMAs of half tile g - 1 from
// the other buffer}, with the eight load instructions of half tile g + 3 spread between them.  The
// fragment reads are inline assembly with explicit waits: the compiler would otherwise wait for every
// outstanding LDS-bound load before any LDS read.
//
// Unit-barrier variant of that schedule (UB, used by the gate/up projection): one wait and one barrier per pair of
// half tiles.  At the start of even iteration g the pair (g, g + 1) has landed and every wave has finished reading
// (g - 2, g - 1), whose two stages take the sixteen load instructions of (g + 2, g + 3), all issued during
// iteration g: half the barriers, for a prefetch distance of two half tiles instead of three.
//
// Operand layout.  Row-major operands are fetched as 64-byte pieces of 16 rows per instruction, i.e. half
// cache lines; in the k-blocked layout (KB: [K / 32][rows][32] for the activations and for repacked weights)
// a half tile of 256 rows is one contiguous 16 KB block and every instruction reads 1 KB of whole lines,
// which is worth about 10 % of the kernel's time.  The SwiGLU output is then written k-blocked as well.
//
// One workgroup per CU walks its tiles in turn (tile i of a workgroup = id + grid * i, which keeps the
// XCD-contiguous tile order); the half-tile stream simply continues into the next tile, so that only the
// first tile pays an empty pipeline.  A tile's last MFMAs run in the next tile's first iteration; the
// epilogue follows that iteration and uses the LDS stage just read as its staging panel.
#include "vla_internal.h"

#include <type_traits>

namespace {

constexpr int BM = 256, BN = 256, HK = 32;
constexpr int REGION = 256 * HK * 2;     // 16 KB per operand per stage
constexpr int STAGE = 2 * REGION;        // 32 KB
constexpr int NSTAGES = 4;

typedef __attribute__((address_space(3))) void lds_void;
typedef int i32x4_t __attribute__((ext_vector_type(4)));

struct DmaGemmParams {
    const bf16_t *A;
    const bf16_t *W0, *W1, *W2;
    void *C;
    int M, N, K, segN;
    int tiles_m, tiles_n;
    int a_rows;      // k-blocked layout: rows per 32-column block of A (and of the SwiGLU output)
    int w_rows;      // k-blocked layout: rows per 32-column block of each weight matrix
    // EPI_QKV_ROPE
    bf16_t *q_out, *kc, *vc;
    const float2 *table;
    int R, pos0, n_heads, pos_stride, H;
    int seg0;        // EPI_QKV_ROPE: what the first weight segment is (0 = q, k, v follow; 1 = k, v only)
    int group;
    int splits;      // > 1: K is cut into `splits` equal ranges; item = range * tiles + tile, and range r of an
                     // EPI_STORE launch writes its fp32 partial product to C + r * M * N
    int wkb;         // row-major activations with k-blocked (repacked) weights: the decode forwards, whose weight
                     // stream comes from HBM and then moves as whole cache lines (w_rows as in the k-blocked layout)
};

template <int OFF>
__device__ __forceinline__ bf16x8_t lds_read(int addr) {
    i32x4_t v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return __builtin_bit_cast(bf16x8_t, v);
}

// One accumulator element, moved out of its accumulation register exactly where the epilogue consumes it
// (left to the compiler all 256 moves are hoisted to the top of the epilogue and spill the fragments that
// are live across it).
__device__ __forceinline__ float acc_read(const f32x4_t &v, int e) {
    float x;
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(x) : "a"(v[e]));
    return x;
}
__device__ __forceinline__ f32x4_t acc_read4(const f32x4_t &v) {
    f32x4_t o;
#pragma unroll
    for (int e = 0; e < 4; e++) o[e] = acc_read(v, e);
    return o;
}
// The matrix pipe's last results must have landed before the first such move (the assembler text is
// opaque to the compiler's hazard handling).
__device__ __forceinline__ void acc_settle() { asm volatile("s_nop 15\n\ts_nop 15"); }

// Epilogue staging panel of one wave: 16 rows x 128 fp32 = 8 KB, no padding; the 16-byte column block cb
// of row r sits at block cb ^ r, which keeps both the column-wise writes (16 lanes = 16 rows) and the
// row-wise reads free of bank conflicts.
__device__ __forceinline__ float *panel_at(float *panel, int row, int cb) { return panel + row * 128 + ((cb ^ row) << 2); }

// Output of one wave.  Per 16-row activation block i a lane holds row (lane % 16) and, per weight block j
// and register r, column 16 j + 4 (lane / 16) + r.  Each block goes through the panel and leaves as whole
// rows.
template <int EPI, bool KB>
__device__ __forceinline__ void epilogue(f32x4_t (&acc)[8][8], const DmaGemmParams &p, int m0, int tn, int wm, int wn,
                                         int lane, float *panel, size_t c_off) {
    const int l16 = lane & 15, kq = lane >> 4;
    if (EPI == EPI_QKV_ROPE) {
        // the wave's 128 columns are one head of q, k or v (head_dim 128)
        const int n0 = tn * BN + wn * 128;
        const int seg_in = n0 / p.H, head = (n0 - seg_in * p.H) >> 7, seg = seg_in + p.seg0;
#pragma unroll
        for (int i = 0; i < 8; i++) {
            const int mblock = m0 + wm * 128 + i * 16;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < 8; j++) *(f32x4_t *)panel_at(panel, l16, j * 4 + kq) = acc_read4(acc[j][i]);
            if (seg == 2) {
#pragma unroll
                for (int it = 0; it < 4; it++) {
                    const int row = it * 4 + (lane >> 4), c = lane & 15, m = mblock + row;
                    f32x4_t a = *(const f32x4_t *)panel_at(panel, row, 2 * c);
                    f32x4_t b = *(const f32x4_t *)panel_at(panel, row, 2 * c + 1);
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
                for (int it = 0; it < 2; it++) {
                    // q: consecutive lanes take consecutive chunks of a row; k: consecutive positions of a chunk
                    const int item = it * 64 + lane;
                    const int row = (seg == 0) ? (item >> 3) : (item & 15);
                    const int c = (seg == 0) ? (item & 7) : (item >> 4);
                    const int m = mblock + row;
                    f32x4_t lo0 = *(const f32x4_t *)panel_at(panel, row, 2 * c), lo1 = *(const f32x4_t *)panel_at(panel, row, 2 * c + 1);
                    f32x4_t hi0 = *(const f32x4_t *)panel_at(panel, row, 16 + 2 * c), hi1 = *(const f32x4_t *)panel_at(panel, row, 17 + 2 * c);
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
    if (EPI == EPI_SWIGLU) {
        // weight blocks 0..3 are gate rows, 4..7 the matching up rows: 64 output columns per wave
        // row-major [M, N], or k-blocked: column c of row m at ((c / 32) * a_rows + m) * 32 + c % 32
        const int c0 = tn * 128 + wn * 64 + (lane & 7) * 8;
        bf16_t *out = (bf16_t *)p.C + (KB ? (size_t)(c0 >> 5) * p.a_rows * 32 + (c0 & 31) : (size_t)c0);
        const size_t row_stride = KB ? 32 : (size_t)p.N;
#pragma unroll
        for (int i = 0; i < 8; i++) {
            const int mblock = m0 + wm * 128 + i * 16;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const f32x4_t g = acc_read4(acc[j][i]), u = acc_read4(acc[j + 4][i]);
                f32x4_t v;
#pragma unroll
                for (int e = 0; e < 4; e++) v[e] = vla_silu_mul(g[e], u[e]);
                *(f32x4_t *)panel_at(panel, l16, j * 4 + kq) = v;
            }
#pragma unroll
            for (int it = 0; it < 2; it++) {
                const int row = it * 8 + (lane >> 3), c2 = lane & 7, m = mblock + row;
                f32x4_t a = *(const f32x4_t *)panel_at(panel, row, 2 * c2);
                f32x4_t b = *(const f32x4_t *)panel_at(panel, row, 2 * c2 + 1);
                bf16x8_t o;
#pragma unroll
                for (int e = 0; e < 4; e++) { o[e] = (bf16_t)a[e]; o[4 + e] = (bf16_t)b[e]; }
                if (m < p.M) *(bf16x8_t *)(out + (size_t)m * row_stride) = o;
            }
        }
        return;
    }
    // fp32 store, or read-modify-write of the fp32 residual stream: whole 512-byte rows, two rows per instruction,
    // through a buffer descriptor over this wave's 128 x 128 block (rows past M fall outside it: their loads
    // return zero and their stores are dropped, so no clamp and no predicate).  x is read XD 16-row blocks ahead of
    // the block being staged, so that a memory latency is paid once per tile and not once per block.
    const int rows_in = min(128, p.M - (m0 + wm * 128));
    float *wave_out = (float *)p.C + c_off + (size_t)(m0 + wm * 128) * p.N + (size_t)tn * BN + wn * 128;
    __amdgpu_buffer_rsrc_t c_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)wave_out, (short)0, rows_in > 0 ? rows_in * p.N * 4 : 0, 0x00020000);
    const int voff = ((lane >> 5) * p.N + (lane & 31) * 4) * 4;
    const int row2 = 2 * p.N * 4;                      // bytes between the row pairs of consecutive instructions
    constexpr int XD = 2;
    i32x4_t x[XD][8];
    // (the stride passes through an empty assembler statement per block: otherwise all 64 offsets of a tile are
    // computed once, before the main loop, and held in registers across it)
    auto load_x = [&](i32x4_t (&xb)[8], int i) {
        int r2 = row2;
        asm volatile("" : "+v"(r2));
#pragma unroll
        for (int it = 0; it < 8; it++) xb[it] = __builtin_amdgcn_raw_buffer_load_b128(c_rsrc, voff + (i * 8 + it) * r2, 0, 0);
    };
    if (EPI == EPI_RESIDUAL) {
#pragma unroll
        for (int i = 0; i < XD; i++) load_x(x[i], i);
    }
#pragma unroll
    for (int i = 0; i < 8; i++) {
        __builtin_amdgcn_sched_barrier(0);
        int r2 = row2;
        asm volatile("" : "+v"(r2));
#pragma unroll
        for (int j = 0; j < 8; j++) *(f32x4_t *)panel_at(panel, l16, j * 4 + kq) = acc_read4(acc[j][i]);
#pragma unroll
        for (int it = 0; it < 8; it++) {
            const int row = it * 2 + (lane >> 5);
            f32x4_t v = *(const f32x4_t *)panel_at(panel, row, lane & 31);
            if (EPI == EPI_RESIDUAL) {
                const f32x4_t xv = __builtin_bit_cast(f32x4_t, x[i % XD][it]);
#pragma unroll
                for (int e = 0; e < 4; e++) v[e] += xv[e];
            }
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(i32x4_t, v), c_rsrc, voff + (i * 8 + it) * r2, 0, 0);
        }
        if (EPI == EPI_RESIDUAL && i + XD < 8) load_x(x[i % XD], i + XD);
    }
}

template <int EPI, bool KB, bool UB = false>
__global__ void __launch_bounds__(256) gemm_bf16_dma_kernel(DmaGemmParams p) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int t = threadIdx.x, lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int n_tiles = p.tiles_m * p.tiles_n;
    const int n_items = n_tiles * p.splits;
    const int K = p.K;
    const int nh = K / HK / p.splits;            // half tiles per item; even: the host sees to it
    int item = blockIdx.x;
    if (item >= n_items || (nh & 1) || nh < 8) return;      // (the host never launches such a K)

    // ---- load cursor -------------------------------------------------------------------------------------
    // A wave instruction covers 16 tile rows: lane l -> row l / 4, position l % 4 of the 64-byte row, which
    // holds chunk (l % 4) ^ ((row / 2) % 4).  This wave loads tile rows wave * 64 .. + 63 of both operands, four
    // instructions each; SwiGLU tiles interleave 64 gate and 64 up rows per wave of the multiply side, so
    // loading wave w takes 64 rows of W0 (w even) or W1 (w odd).
    const int chunk_off = ((lane & 3) ^ ((lane >> 3) & 3)) << 4;
    const bool WKB = KB ? true : (p.wkb != 0);   // the weights' layout (a compile-time constant in the k-blocked kernels)
    const int row_bytes = KB ? 64 : K * 2;       // distance of consecutive tile rows of one half tile
    const int w_row_bytes = WKB ? 64 : K * 2;
    const int a_thread_off = (wave * 64 + (lane >> 2)) * row_bytes + chunk_off;
    const int w_thread_off = (((EPI == EPI_SWIGLU) ? (wave >> 1) * 64 : wave * 64) + (lane >> 2)) * w_row_bytes + chunk_off;
    const int tile_bytes = BM * K * 2;
    // distance of consecutive half tiles: 64 bytes along the row, or one 32-column block of all rows
    const unsigned a_half = KB ? (unsigned)p.a_rows * 64u : 64u, w_half = WKB ? (unsigned)p.w_rows * 64u : 64u;
    __amdgpu_buffer_rsrc_t a_rsrc, w_rsrc;
    int ld_item, ld_h;
    int nx_tm, nx_tn, nx_split;
    auto setup_load = [&](int it) {
        int tm, tn;
        const int split = __builtin_amdgcn_readfirstlane(it / n_tiles);
        vla_tile_of_block(it - split * n_tiles, p.tiles_m, p.tiles_n, tm, tn, p.group);
        // first element of this item's K range within a row panel: k-blocked, whole 32-column blocks; row-major, columns
        const size_t a_k0 = KB ? (size_t)split * nh * (a_half / 2) : (size_t)split * nh * HK;
        const size_t w_k0 = WKB ? (size_t)split * nh * (w_half / 2) : (size_t)split * nh * HK;
        if (KB) a_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)(p.A + (size_t)tm * BM * 32 + a_k0), (short)0, (int)((unsigned)(nh - 1) * a_half + 16384u), 0x00020000);
        else a_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)(p.A + (size_t)tm * BM * K + a_k0), (short)0, tile_bytes, 0x00020000);
        if (EPI == EPI_SWIGLU) {
            const bf16_t *Wp = (wave & 1) ? p.W1 : p.W0;
            if (WKB) w_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)(Wp + (size_t)(tn * 128) * 32 + w_k0), (short)0, (int)((unsigned)(nh - 1) * w_half + 8192u), 0x00020000);
            else w_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)(Wp + (size_t)(tn * 128) * K + w_k0), (short)0, tile_bytes / 2, 0x00020000);
        } else {
            const int n = tn * BN;
            const int seg = __builtin_amdgcn_readfirstlane(n / p.segN);
            const bf16_t *Wp = seg == 0 ? p.W0 : (seg == 1 ? p.W1 : p.W2);
            if (WKB) w_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)(Wp + (size_t)(n - seg * p.segN) * 32 + w_k0), (short)0, (int)((unsigned)(nh - 1) * w_half + 16384u), 0x00020000);
            else w_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)(Wp + (size_t)(n - seg * p.segN) * K + w_k0), (short)0, tile_bytes, 0x00020000);
        }
        ld_item = it;
        ld_h = 0;
        nx_tm = tm; nx_tn = tn; nx_split = split;
    };
    // instruction pair i (0..3) of the cursor's half tile into LDS stage `stage`
    auto dma = [&](int stage, int i) {
        char *base = lds + stage * STAGE + wave * 4096 + i * 1024;
        const int blk = i * 16 * row_bytes, w_blk = i * 16 * w_row_bytes;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, (lds_void *)base, 16, a_thread_off, (int)((unsigned)ld_h * a_half) + blk, 0, 0);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(w_rsrc, (lds_void *)(base + REGION), 16, w_thread_off, (int)((unsigned)ld_h * w_half) + w_blk, 0, 0);
    };
    // next half tile, else the next item's first, else stay (the last half tile is fetched again, never used)
    auto advance = [&]() {
        ld_h++;
        if (ld_h == nh) {
            const int nxt = ld_item + (int)gridDim.x;
            if (nxt < n_items) setup_load(nxt);
            else ld_h--;
        }
    };

    // ---- fragments -----------------------------------------------------------------------------------------
    const int l16 = lane & 15, kq = lane >> 4, fsw = (l16 >> 1) & 3;
    const int lds0 = (int)(size_t)(lds_void *)lds;
    const int a_base = lds0 + (wm * 128 + l16) * 64 + ((kq ^ fsw) << 4);
    const int w_base = lds0 + REGION + (wn * 128 + l16) * 64 + ((kq ^ fsw) << 4);
    f32x4_t acc[8][8];                  // [weight block][activation block]
    bf16x8_t af[2][8], wf[2][8];
#pragma unroll
    for (int b = 0; b < 2; b++)
#pragma unroll
        for (int i = 0; i < 8; i++)
#pragma unroll
            for (int e = 0; e < 8; e++) { af[b][i][e] = (bf16_t)0.f; wf[b][i][e] = (bf16_t)0.f; }
    auto zero_acc = [&]() {
#pragma unroll
        for (int j = 0; j < 8; j++)
#pragma unroll
            for (int i = 0; i < 8; i++)
#pragma unroll
                for (int r = 0; r < 4; r++) acc[j][i][r] = 0.f;
    };
    zero_acc();

#define VLA_SB() __builtin_amdgcn_sched_barrier(0)
#define VLA_Q(n) std::integral_constant<int, n> {}
    // group q (0..15): fragment reads into buffer B and four MFMAs from buffer B ^ 1 (weight block q / 2,
    // activation blocks 4 (q % 2) .. + 3).  Fragment f (0..15; even: weight block f / 2, odd: activation block
    // f / 2) is read in group f / 2 for f < 8 and in group f - 4 after that: all reads are issued by group 11,
    // so that the last sixteen MFMAs cover their latency before the end-of-iteration wait.
    auto read_frag = [&](auto b_c, auto f_c, int soff) {
        constexpr int B = decltype(b_c)::value, f = decltype(f_c)::value;
        constexpr int blk = f >> 1;
        if (f & 1) af[B][blk] = lds_read<blk * 1024>(a_base + soff);
        else wf[B][blk] = lds_read<blk * 1024>(w_base + soff);
    };
    auto group = [&](auto b_c, auto q_c, int soff) {
        constexpr int B = decltype(b_c)::value, q = decltype(q_c)::value;
        if (q < 4) {
            read_frag(b_c, std::integral_constant<int, (q < 4 ? 2 * q : 0)>{}, soff);
            read_frag(b_c, std::integral_constant<int, (q < 4 ? 2 * q + 1 : 0)>{}, soff);
        } else if (q < 12) {
            read_frag(b_c, std::integral_constant<int, (q >= 4 && q < 12 ? q + 4 : 0)>{}, soff);
        }
        constexpr int j = q >> 1, i0 = (q & 1) * 4;
#pragma unroll
        for (int i = i0; i < i0 + 4; i++)
            acc[j][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[B ^ 1][j], af[B ^ 1][i], acc[j][i], 0, 0, 0);
    };
    // this wave's fragment reads have landed; the fragments pass through so that no MFMA moves above the wait
    auto wait_frags = [&](int B) {
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(af[B][0]), "+v"(af[B][1]), "+v"(af[B][2]), "+v"(af[B][3]), "+v"(af[B][4]), "+v"(af[B][5]),
                       "+v"(af[B][6]), "+v"(af[B][7]), "+v"(wf[B][0]), "+v"(wf[B][1]), "+v"(wf[B][2]), "+v"(wf[B][3]),
                       "+v"(wf[B][4]), "+v"(wf[B][5]), "+v"(wf[B][6]), "+v"(wf[B][7]));
    };
    // iteration g of the workgroup's half-tile stream: reads half tile g into buffer b, multiplies half tile
    // g - 1 from the other buffer, and (unless `defer`) issues the loads of half tile g + 3
    auto iteration = [&](auto b_c, int g, bool defer) {
        const int soff = (g & 3) * STAGE, sn = (g + 3) & 3;
        // vmcnt counts in issue order: at most the 16 load instructions of half tiles g + 1 and g + 2 may still be
        // in flight (right after an epilogue this also waits for the epilogue's own stores)
        asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        asm volatile("s_barrier" ::: "memory");   // everyone's loads of g have landed, everyone's reads of g - 1 are done
        VLA_SB();
        group(b_c, VLA_Q(0), soff); VLA_SB();
        group(b_c, VLA_Q(1), soff); VLA_SB();
        if (!defer) dma(sn, 0);
        VLA_SB();
        group(b_c, VLA_Q(2), soff); VLA_SB();
        group(b_c, VLA_Q(3), soff); VLA_SB();
        group(b_c, VLA_Q(4), soff); VLA_SB();
        group(b_c, VLA_Q(5), soff); VLA_SB();
        if (!defer) dma(sn, 1);
        VLA_SB();
        group(b_c, VLA_Q(6), soff); VLA_SB();
        group(b_c, VLA_Q(7), soff); VLA_SB();
        group(b_c, VLA_Q(8), soff); VLA_SB();
        group(b_c, VLA_Q(9), soff); VLA_SB();
        if (!defer) dma(sn, 2);
        VLA_SB();
        group(b_c, VLA_Q(10), soff); VLA_SB();
        group(b_c, VLA_Q(11), soff); VLA_SB();
        group(b_c, VLA_Q(12), soff); VLA_SB();
        group(b_c, VLA_Q(13), soff); VLA_SB();
        if (!defer) { dma(sn, 3); advance(); }
        VLA_SB();
        group(b_c, VLA_Q(14), soff); VLA_SB();
        group(b_c, VLA_Q(15), soff); VLA_SB();
        wait_frags(decltype(b_c)::value);
        VLA_SB();
    };

    using B0 = std::integral_constant<int, 0>;
    using B1 = std::integral_constant<int, 1>;
    if constexpr (UB) {
        // Unit-barrier schedule: one wait and one barrier per pair of half tiles.  At the start of even iteration g
        // half tiles g and g + 1 have landed and every wave has finished reading g - 2 and g - 1, whose stages take
        // the loads of g + 2 and g + 3, all issued during iteration g.
        auto iteration_ub = [&](auto b_c, int g, bool defer) {
            constexpr int B = decltype(b_c)::value;
            const int soff = (g & 3) * STAGE, s2 = (g + 2) & 3, s3 = (g + 3) & 3;
            if (B == 0) {
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                asm volatile("s_barrier" ::: "memory");
            }
            VLA_SB();
            group(b_c, VLA_Q(0), soff); VLA_SB();
            group(b_c, VLA_Q(1), soff); VLA_SB();
            if (B == 0 && !defer) dma(s2, 0);
            VLA_SB();
            group(b_c, VLA_Q(2), soff); VLA_SB();
            group(b_c, VLA_Q(3), soff); VLA_SB();
            if (B == 0 && !defer) dma(s2, 1);
            VLA_SB();
            group(b_c, VLA_Q(4), soff); VLA_SB();
            group(b_c, VLA_Q(5), soff); VLA_SB();
            if (B == 0 && !defer) dma(s2, 2);
            VLA_SB();
            group(b_c, VLA_Q(6), soff); VLA_SB();
            group(b_c, VLA_Q(7), soff); VLA_SB();
            if (B == 0 && !defer) { dma(s2, 3); advance(); }
            VLA_SB();
            group(b_c, VLA_Q(8), soff); VLA_SB();
            group(b_c, VLA_Q(9), soff); VLA_SB();
            if (B == 0 && !defer) dma(s3, 0);
            VLA_SB();
            group(b_c, VLA_Q(10), soff); VLA_SB();
            group(b_c, VLA_Q(11), soff); VLA_SB();
            if (B == 0 && !defer) dma(s3, 1);
            VLA_SB();
            group(b_c, VLA_Q(12), soff); VLA_SB();
            group(b_c, VLA_Q(13), soff); VLA_SB();
            if (B == 0 && !defer) dma(s3, 2);
            VLA_SB();
            group(b_c, VLA_Q(14), soff); VLA_SB();
            group(b_c, VLA_Q(15), soff); VLA_SB();
            if (B == 0 && !defer) { dma(s3, 3); advance(); }
            VLA_SB();
            wait_frags(B);
            VLA_SB();
        };
        setup_load(item);
        int tm = nx_tm, tn = nx_tn, split = nx_split;
#pragma unroll
        for (int d = 0; d < 2; d++) {
#pragma unroll
            for (int i = 0; i < 4; i++) dma(d, i);
            advance();
        }
        const int n_mine = (n_items - item + (int)gridDim.x - 1) / (int)gridDim.x;
        const int g_end = n_mine * nh;
        int next_done = nh;
        for (int g = 0;; g += 2) {
            const bool boundary = (g == next_done);
            iteration_ub(B0{}, g, boundary && g != g_end);
            if (boundary) {
                asm volatile("s_barrier" ::: "memory");
                acc_settle();
                float *panel = (float *)(lds + (g & 3) * STAGE) + wave * (16 * 128);
                epilogue<EPI, KB>(acc, p, tm * BM, tn, wm, wn, lane, panel, (size_t)split * p.M * p.N);
                if (g == g_end) break;
                zero_acc();
                // the loads this boundary iteration held back (half tiles g + 2 and g + 3, both of the next item)
#pragma unroll
                for (int i = 0; i < 4; i++) dma((g + 2) & 3, i);
                advance();
#pragma unroll
                for (int i = 0; i < 4; i++) dma((g + 3) & 3, i);
                advance();
                tm = nx_tm; tn = nx_tn; split = nx_split;
                next_done += nh;
            }
            iteration_ub(B1{}, g + 1, false);
        }
    } else {
    setup_load(item);
    int tm = nx_tm, tn = nx_tn, split = nx_split;
#pragma unroll
    for (int d = 0; d < 3; d++) {
#pragma unroll
        for (int i = 0; i < 4; i++) dma(d, i);
        advance();
    }
    // Half tile h of the workgroup's n-th item is stream element g = n * nh + h; it is read in iteration g and
    // multiplied in iteration g + 1, so an item is complete after the first iteration of the next one (or after
    // one extra iteration at the end of the stream).  nh is even, so that iteration is always an even one.
    int n_mine = (n_items - item + (int)gridDim.x - 1) / (int)gridDim.x;
    const int g_end = n_mine * nh;
    int next_done = nh;                          // the even iteration after which the current item is complete
    for (int g = 0;; g += 2) {
        const bool boundary = (g == next_done);
        iteration(B0{}, g, boundary && g != g_end);
        if (boundary) {
            // every wave is done reading stage g % 4: it becomes the panel
            asm volatile("s_barrier" ::: "memory");
            acc_settle();
            float *panel = (float *)(lds + (g & 3) * STAGE) + wave * (16 * 128);
            epilogue<EPI, KB>(acc, p, tm * BM, tn, wm, wn, lane, panel, (size_t)split * p.M * p.N);
            if (g == g_end) break;
            zero_acc();
            tm = nx_tm; tn = nx_tn; split = nx_split;   // the cursor moved on to the next item four iterations ago
            next_done += nh;
            const int sn = (g + 3) & 3;          // the loads this boundary iteration held back
#pragma unroll
            for (int i = 0; i < 4; i++) dma(sn, i);
            advance();
        }
        iteration(B1{}, g + 1, false);
    }
    }
}

template <int EPI, bool KB, bool UB = false>
int launch_plain(const DmaGemmParams &p, hipStream_t st) {
    static bool attr_set = false;
    static int n_cu = 0;
    const size_t lds = NSTAGES * (size_t)STAGE;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)gemm_bf16_dma_kernel<EPI, KB, UB>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) {
            vla_set_error("hipFuncSetAttribute(gemm_bf16_dma) failed: %s", hipGetErrorString(e));
            return VLA_EHIP;
        }
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1) {
            vla_set_error("gemm_bf16_dma: cannot read the compute-unit count");
            return VLA_EHIP;
        }
        attr_set = true;
    }
    // one workgroup per CU (128 KB of LDS, 512 registers per lane); blockIdx % 8 is the XCD, and a stride of a
    // multiple of 8 keeps every workgroup's items on its own XCD's share of the tile order
    const int n_items = p.tiles_m * p.tiles_n * p.splits;
    int grid = n_items;
    if (n_cu % 8 == 0 && n_items > n_cu) grid = n_cu;
    gemm_bf16_dma_kernel<EPI, KB, UB><<<grid, 256, lds, st>>>(p);
    int rc = vla_check_launch("gemm_bf16_dma");
    return rc ? rc : 1;
}

template <int EPI, bool KB, bool UB = false>
int launch(const DmaGemmParams &p, hipStream_t st) {
    const double flops = 2.0 * p.M * p.K * (EPI == EPI_SWIGLU ? 2.0 * p.N : (double)p.N);
    ProfScope ps(EPI == EPI_SWIGLU ? "gemm_bf16_dma<swiglu>" : EPI == EPI_RESIDUAL ? "gemm_bf16_dma<residual>"
                 : EPI == EPI_QKV_ROPE ? "gemm_bf16_dma<qkv_rope>" : "gemm_bf16_dma<store>", flops, st);
    return launch_plain<EPI, KB, UB>(p, st);
}

template <int EPI>
int launch_kb(const DmaGemmParams &p, bool kb, hipStream_t st) {
    // The unit-barrier schedule pays for the gate/up projection (3.7 % faster at M = 73728: 10.03 against 10.41 ms);
    // the QKV and down projections run the same with either and the O projection, whose short tiles end in the
    // heaviest epilogue, 5 % slower.
    if constexpr (EPI == EPI_SWIGLU) {
        if (kb) return launch<EPI, true, true>(p, st);
    }
    return kb ? launch<EPI, true>(p, st) : launch<EPI, false>(p, st);
}

}  // namespace

// Handles bf16 problems with K a multiple of 64 and at least 256 (the cursor must never be more than one item
// ahead of the multiply side), N tiles that do not straddle weight segments, and an activation buffer that
// covers whole 256-row tiles.  With g.kblocked the activations (a_rows rows per 32-column block), the weights
// (segN + pad rows per block, each segment repacked on its own) and a SwiGLU output are in the k-blocked layout.
// Returns 1 if handled, 0 if declined, < 0 on a launch error.
int try_gemm_bf16_dma(const GemmArgs &g, hipStream_t st) {
    if (g.M < 1 || g.K % 64 != 0 || g.K < 256 || g.a_rows < (g.M + BM - 1) / BM * BM) return 0;
    const bool kb = g.kblocked != 0;
    if (kb && ((size_t)g.a_rows * g.K * 2 >= ((size_t)1 << 31) || (size_t)(g.segN + VLA_KB_PAD_ROWS) * g.K * 2 >= ((size_t)1 << 31))) return 0;
    DmaGemmParams p{};
    p.A = (const bf16_t *)g.A;
    p.W0 = (const bf16_t *)g.W[0]; p.W1 = (const bf16_t *)g.W[1]; p.W2 = (const bf16_t *)g.W[2];
    p.C = g.C; p.M = g.M; p.K = g.K; p.segN = g.segN;
    p.a_rows = g.a_rows; p.w_rows = g.segN + VLA_KB_PAD_ROWS;
    p.splits = 1;
    {
        // tile rows per column panel of the walk: 4, except for the QKV projection (1.9 % faster with 2 at
        // M = 73728: 5.73 against 5.84 ms; the other projections within 0.5 % either way)
        p.group = g.epilogue == EPI_QKV_ROPE ? 2 : 4;
    }
    p.tiles_m = (g.M + BM - 1) / BM;
    if (g.epilogue == EPI_SWIGLU) {
        if (g.segN % 128 != 0) return 0;
        p.N = g.segN;
        p.tiles_n = g.segN / 128;
        return launch_kb<EPI_SWIGLU>(p, kb, st);
    }
    if (g.segN % BN != 0) return 0;
    if (g.epilogue == EPI_QKV_ROPE) {
        const QkvRopeArgs *ra = g.rope;
        if (!ra || ra->kv->d != 128 || (g.n_seg != 3 && g.n_seg != 2) || g.segN != ra->kv->n_heads * 128) return 0;
        if (g.n_seg == 3 && !ra->q_out) return 0;
        p.seg0 = 3 - g.n_seg;                   // two segments: the k and v projections alone
        p.q_out = (bf16_t *)ra->q_out;
        p.kc = (bf16_t *)ra->kv->k + (size_t)ra->layer * ra->kv->layer_elems;
        p.vc = (bf16_t *)ra->kv->v + (size_t)ra->layer * ra->kv->layer_elems;
        p.table = ra->table;
        p.R = ra->rows->R; p.pos0 = ra->rows->pos0; p.n_heads = ra->kv->n_heads;
        p.pos_stride = ra->kv->pos_stride; p.H = g.segN;
        p.N = g.n_seg * g.segN;
        p.tiles_n = p.N / BN;
        return launch_kb<EPI_QKV_ROPE>(p, kb, st);
    }
    p.N = g.n_seg * g.segN;
    p.tiles_n = p.N / BN;
    return g.epilogue == EPI_RESIDUAL ? launch_kb<EPI_RESIDUAL>(p, kb, st) : launch_kb<EPI_STORE>(p, kb, st);
}

// Split-K form for forwards of at most 256 rows (one tile row): the K range is cut into 2, 4 or 8 equal parts so
// that tiles x parts workgroups are busy, each part's fp32 product goes to `scratch` ([parts][M][N], for SwiGLU
// N = gate columns then up columns) and launch_splitk_reduce adds the parts in order and applies the epilogue.
// Takes the QKV projection (fp32 output) and the gate/up projection; declines everything else, and problems
// where no such split leaves at least a fifth of the CUs more busy than without it.  Row-major operands.
int try_gemm_bf16_dma_splitk(const GemmArgs &g, void *scratch, size_t scratch_bytes, hipStream_t st) {
    if (g.kblocked || g.M < 1 || g.M > BM || g.a_rows < BM || g.K % 64 != 0 || !scratch) return 0;
    if (g.epilogue != EPI_STORE && g.epilogue != EPI_SWIGLU) return 0;
    if (g.segN % BN != 0) return 0;
    static int n_cu = 0;
    if (!n_cu) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1) {
            vla_set_error("gemm_bf16_dma: cannot read the compute-unit count");
            return VLA_EHIP;
        }
    }
    const int n_seg = g.epilogue == EPI_SWIGLU ? 2 : g.n_seg;
    const int N = n_seg * g.segN, tiles = N / BN, nh = g.K / HK;
    int splits = 1;
    while (splits < 8 && tiles * splits * 2 <= n_cu && (nh / (splits * 2)) % 2 == 0 && nh / (splits * 2) >= 8 &&
           nh % (splits * 2) == 0 && (size_t)(splits * 2) * g.M * N * sizeof(float) <= scratch_bytes)
        splits *= 2;
    if (splits < 2 || tiles * splits * 5 < n_cu * 3) return 0;
    DmaGemmParams p{};
    p.A = (const bf16_t *)g.A;
    p.W0 = (const bf16_t *)g.W[0]; p.W1 = (const bf16_t *)g.W[1]; p.W2 = (const bf16_t *)g.W[2];
    p.C = scratch; p.M = g.M; p.K = g.K; p.segN = g.segN;
    p.a_rows = g.a_rows; p.w_rows = 0; p.group = 4; p.splits = splits;
    p.tiles_m = 1; p.N = N; p.tiles_n = tiles;
    // repacked copies of the weights, where the caller has them and the 32-bit offsets of the loads cover a segment
    bool have_kb = g.Wkb[0] && (size_t)(g.segN + VLA_KB_PAD_ROWS) * g.K * 2 < ((size_t)1 << 31);
    for (int i = 1; i < n_seg; i++) have_kb = have_kb && g.Wkb[i];
    if (have_kb) {
        p.W0 = (const bf16_t *)g.Wkb[0]; p.W1 = (const bf16_t *)g.Wkb[1]; p.W2 = (const bf16_t *)g.Wkb[2];
        p.w_rows = g.segN + VLA_KB_PAD_ROWS; p.wkb = 1;
    }
    int rc;
    {
        ProfScope ps(g.epilogue == EPI_SWIGLU ? "gemm_dma_splitk<swiglu>" : "gemm_dma_splitk<store>", 2.0 * g.M * g.K * (double)N, st);
        rc = launch_plain<EPI_STORE, false>(p, st);
        if (rc != 1) return rc;
    }
    if (g.deferred_splits && g.epilogue == EPI_STORE) *g.deferred_splits = splits;
    else if ((rc = launch_splitk_reduce(g.epilogue, g.C, (const float *)scratch, splits, g.M, g.epilogue == EPI_SWIGLU ? g.segN : N, st))) return rc;
    return 1;
}

// Split-K form for multi-row problems with few output tiles (the LoRA-gradient products: 256 output columns, or a
// contraction over all rows of a micro-batch): the K range is cut into `parts` equal ranges so that tiles x parts
// items keep the CUs busy, each range's fp32 product goes to `scratch` ([parts][M][N]) and launch_splitk_reduce adds
// them in order.  Row-major operands, fp32 output only.  `parts` minimises a cost estimate (below); declines (0) when
// that leaves one part or the scratch is too small.
int try_gemm_bf16_dma_splitk_rows(const GemmArgs &g, void *scratch, size_t scratch_bytes, hipStream_t st) {
    if (g.kblocked || g.epilogue != EPI_STORE || g.M < 1 || g.K % 64 != 0 || g.K < 256 || !scratch) return 0;
    if (g.segN % BN != 0 || g.a_rows < (g.M + BM - 1) / BM * BM) return 0;
    static int n_cu = 0;
    if (!n_cu) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1) {
            vla_set_error("gemm_bf16_dma: cannot read the compute-unit count");
            return VLA_EHIP;
        }
    }
    const int N = g.n_seg * g.segN, tiles_m = (g.M + BM - 1) / BM, tiles = tiles_m * (N / BN), nh = g.K / HK;
    // cost in half-tile times (about 0.8 us): rounds of items x (half tiles per item + about 8 for an item's prologue
    // and fp32 epilogue), plus the reduction's traffic (0.5 MB written and read per tile and part, about 0.16)
    auto cost_of = [&](int parts) {
        const long rounds = (tiles * parts + n_cu - 1) / n_cu;
        return rounds * (nh / parts + 8) * 100 + (parts > 1 ? 16L * parts * tiles : 0);
    };
    int best = 1;
    long best_cost = cost_of(1);
    for (int parts = 2; parts <= 32; parts++) {
        const int per = nh / parts;
        if (nh % parts != 0 || (per & 1) || per < 8) continue;
        if ((size_t)parts * g.M * N * sizeof(float) > scratch_bytes) break;
        const long cost = cost_of(parts);
        if (cost < best_cost) { best_cost = cost; best = parts; }
    }
    if (best < 2) return 0;
    DmaGemmParams p{};
    p.A = (const bf16_t *)g.A;
    p.W0 = (const bf16_t *)g.W[0]; p.W1 = (const bf16_t *)g.W[1]; p.W2 = (const bf16_t *)g.W[2];
    p.C = scratch; p.M = g.M; p.K = g.K; p.segN = g.segN;
    p.a_rows = g.a_rows; p.w_rows = 0; p.group = 4; p.splits = best;
    p.tiles_m = tiles_m; p.N = N; p.tiles_n = N / BN;
    {
        ProfScope ps("gemm_dma_splitk_rows<store>", 2.0 * g.M * g.K * (double)N, st);
        const int rc = launch_plain<EPI_STORE, false>(p, st);
        if (rc != 1) return rc;
    }
    const int rc = launch_splitk_reduce(EPI_STORE, g.C, (const float *)scratch, best, g.M, N, st);
    return rc ? rc : 1;
}

namespace {

// Repack of one weight matrix [N, K] into [K / 32][N + pad][32]: a thread moves one 16-byte piece (the pad rows
// are never read).
__global__ void __launch_bounds__(256) weight_kblock_kernel(bf16_t *dst, const bf16_t *src, int N, int K) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;       // (n, 8-column piece)
    const int pieces = K / 8;
    if (idx >= (size_t)N * pieces) return;
    const int n = (int)(idx / pieces), pc = (int)(idx - (size_t)n * pieces);
    const bf16x8_t v = *(const bf16x8_t *)(src + (size_t)n * K + pc * 8);
    *(bf16x8_t *)(dst + ((size_t)(pc >> 2) * (N + VLA_KB_PAD_ROWS) + n) * 32 + (pc & 3) * 8) = v;
}

}  // namespace

int launch_weight_kblock(bf16_t *dst, const bf16_t *src, int N, int K, hipStream_t st) {
    if (K % 32 != 0) { vla_set_error("weight repack: K = %d is not a multiple of 32", K); return VLA_ESHAPE; }
    const size_t total = (size_t)N * (K / 8);
    if (total == 0) return 0;
    weight_kblock_kernel<<<(unsigned)((total + 255) / 256), 256, 0, st>>>(dst, src, N, K);
    return vla_check_launch("weight_kblock");
}
