// bf16 GEMM for single-row (decode) forwards with 129..256 rows: C[M, N] = A[M, K] . W[N, K]^T.
//
// At these sizes the weights are read once from HBM and the job is to keep that stream busy while the
// whole activation matrix is re-read (from L2) by every workgroup.  A workgroup therefore takes all M
// rows, a narrow block of 64 weight rows and one K range: compared with the 256 x 256 tile this cuts
// the fp32 partial sums that split K has to write and re-read by a factor of four at equal workgroup
// count, and two workgroups fit a CU (80 KB of LDS, < 256 registers), each hiding the other's barriers
// and load latency.  Partial sums leave as whole rows and are reduced in split order by the decode
// GEMM's reduction kernel (no atomics), which also applies the epilogue.
//
// LDS stage: activation tile BM x 64 and weight tile 64 x 64 bf16, rows of eight 16-byte chunks with
// chunk c of row r at position c ^ ((r >> 1) & 7); global loads are buffer loads with one per-thread
// offset (row t / 8 of a 32-row block, chunk t % 8) plus scalar block and K offsets.
#include "vla_internal.h"

#include <type_traits>

namespace {

constexpr int BK = 64, BN = 64;
constexpr int W_BYTES = BN * BK * 2;

struct MidParams {
    const bf16_t *A;
    const bf16_t *W0, *W1, *W2;
    float *P;        // [splits][M][NP] fp32 partial sums (SwiGLU: NP = 2N, gate columns then up columns)
    int M, N, K, segN;
    int n_tiles, splits;
};

__device__ __forceinline__ int swz(int row) { return (row >> 1) & 7; }

constexpr int PANEL_LD = 68;     // floats per staged row of the output panel (64 + pad)

template <int BM, int EPI>
__global__ void __launch_bounds__(256, 2) gemm_mid_kernel(MidParams p) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    constexpr int A_BYTES = BM * BK * 2;
    constexpr int STAGE = A_BYTES + W_BYTES;
    constexpr int RB = BM / 128;            // 32-row activation blocks per wave
    constexpr int ACH = BM / 32;            // 16-byte activation chunks a thread loads per K tile
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int K = p.K;
    const int split = blockIdx.x / p.n_tiles, tile = blockIdx.x - split * p.n_tiles;
    const int ktiles = K / BK;
    const int kt0 = (int)((long)split * ktiles / p.splits), kt1 = (int)((long)(split + 1) * ktiles / p.splits);

    const int trow = t >> 3;
    const int thread_off = trow * K * 2 + ((t & 7) ^ swz(trow)) * 16;
    const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)p.A, (short)0, BM * K * 2, 0x00020000);
    __amdgpu_buffer_rsrc_t w_rsrc0, w_rsrc1;
    if (EPI == EPI_SWIGLU) {           // 32 gate rows then 32 up rows
        w_rsrc0 = __builtin_amdgcn_make_buffer_rsrc((void *)(p.W0 + (size_t)tile * 32 * K), (short)0, 32 * K * 2, 0x00020000);
        w_rsrc1 = __builtin_amdgcn_make_buffer_rsrc((void *)(p.W1 + (size_t)tile * 32 * K), (short)0, 32 * K * 2, 0x00020000);
    } else {
        const int n = tile * BN;
        const int seg = n / p.segN;
        const bf16_t *Wp = seg == 0 ? p.W0 : (seg == 1 ? p.W1 : p.W2);
        w_rsrc0 = __builtin_amdgcn_make_buffer_rsrc((void *)(Wp + (size_t)(n - seg * p.segN) * K), (short)0, 32 * K * 2, 0x00020000);
        w_rsrc1 = __builtin_amdgcn_make_buffer_rsrc((void *)(Wp + (size_t)(n - seg * p.segN + 32) * K), (short)0, 32 * K * 2, 0x00020000);
    }

    // Three register sets of staged loads: the loads of K tile kt + 3 are issued while tile kt is
    // multiplied, so about three tiles (120 KB per workgroup at 256 rows) are in flight per workgroup --
    // most of it activation re-reads from L2, which is what bounds the weight stream here.
    bf16x8_t stage_a[3][ACH], stage_w[3][2];
    auto gload = [&](auto set_c, int kt) {
        constexpr int SET = decltype(set_c)::value;
        const int ko = kt * BK * 2;
#pragma unroll
        for (int i = 0; i < ACH; i++)
            stage_a[SET][i] = __builtin_bit_cast(bf16x8_t, __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, thread_off, ko + i * 32 * K * 2, 0));
        stage_w[SET][0] = __builtin_bit_cast(bf16x8_t, __builtin_amdgcn_raw_buffer_load_b128(w_rsrc0, thread_off, ko, 0));
        stage_w[SET][1] = __builtin_bit_cast(bf16x8_t, __builtin_amdgcn_raw_buffer_load_b128(w_rsrc1, thread_off, ko, 0));
    };
    auto lstore = [&](auto set_c, int s) {
        constexpr int SET = decltype(set_c)::value;
        char *base = lds + s * STAGE;
#pragma unroll
        for (int i = 0; i < ACH; i++) *(bf16x8_t *)(base + (i * 256 + t) * 16) = stage_a[SET][i];
#pragma unroll
        for (int i = 0; i < 2; i++) *(bf16x8_t *)(base + A_BYTES + (i * 256 + t) * 16) = stage_w[SET][i];
    };

    // fragment rows: the wave's activation rows and all 64 weight rows
    int a_off[RB], w_off[2];
    const int l32 = lane & 31, khalf = lane >> 5;
    const int fsw = swz(l32);            // block starts are multiples of 32 rows: the swizzle depends on l32 only
#pragma unroll
    for (int i = 0; i < RB; i++) a_off[i] = (wave * (BM / 4) + i * 32 + l32) * 128;
#pragma unroll
    for (int j = 0; j < 2; j++) w_off[j] = A_BYTES + (j * 32 + l32) * 128;

    f32x16_t acc[2][RB];
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
        for (int i = 0; i < RB; i++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[j][i][r] = 0.f;

    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;
    using S2 = std::integral_constant<int, 2>;
    const int last = kt1 - 1;
    // tile kt0 + n lives in register set n % 3 until it is written to LDS stage n % 2 during tile n - 1;
    // past the end the last tile is fetched again and never used (no branch around the loads)
    gload(S0{}, kt0);
    gload(S1{}, min(kt0 + 1, last));
    gload(S2{}, min(kt0 + 2, last));
    lstore(S0{}, 0);
    __syncthreads();
    int n = 0;                                             // tiles done
    auto ktile = [&](auto set_c, int kt) {
        // set_c: the set that held this tile (free now: takes tile kt + 3); the next tile sits in set + 1
        constexpr int SET = decltype(set_c)::value;
        using Next = std::integral_constant<int, (SET + 1) % 3>;
        const int s = n & 1;
        const char *base = lds + s * STAGE;
        gload(set_c, min(kt + 3, last));
#pragma unroll
        for (int ks = 0; ks < 4; ks++) {
            const int c = ((ks * 2 + khalf) ^ fsw) << 4;
            bf16x8_t af[RB], wf[2];
#pragma unroll
            for (int i = 0; i < RB; i++) af[i] = *(const bf16x8_t *)(base + a_off[i] + c);
#pragma unroll
            for (int j = 0; j < 2; j++) wf[j] = *(const bf16x8_t *)(base + w_off[j] + c);
#pragma unroll
            for (int j = 0; j < 2; j++)
#pragma unroll
                for (int i = 0; i < RB; i++)
                    acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[j], af[i], acc[j][i], 0, 0, 0);
        }
        lstore(Next{}, s ^ 1);
        __syncthreads();           // stage s is free for the tile after next, stage s ^ 1 is complete
        n++;
    };
    for (int kt = kt0; kt < kt1; kt += 3) {
        ktile(S0{}, kt);
        if (kt + 1 < kt1) ktile(S1{}, kt + 1);
        if (kt + 2 < kt1) ktile(S2{}, kt + 2);
    }

    // ---- partial sums out: each 32 x 64 block through a per-wave LDS panel, then whole 256-byte rows ----
    // A lane holds activation row l32 of the block and, per accumulator register r of weight block j,
    // output column 32 j + 8 (r / 4) + 4 khalf + r % 4.
    float *panel = (float *)lds + wave * (32 * PANEL_LD);
    const int NP = (EPI == EPI_SWIGLU) ? 2 * p.N : p.N;
    const int c4 = (lane & 15) * 4;                         // column of this lane's 16-byte piece of a row
    int col;
    if (EPI == EPI_SWIGLU) col = (c4 < 32 ? 0 : p.N - 32) + tile * 32 + c4;       // columns 32..63 are the up half
    else col = tile * BN + c4;
    float *out = p.P + (size_t)split * p.M * NP + col;
#pragma unroll
    for (int i = 0; i < RB; i++) {
        const int mblock = wave * (BM / 4) + i * 32;
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
                f32x4_t v;
#pragma unroll
                for (int e = 0; e < 4; e++) v[e] = acc[j][i][g * 4 + e];
                *(f32x4_t *)(panel + l32 * PANEL_LD + j * 32 + g * 8 + 4 * khalf) = v;
            }
#pragma unroll
        for (int it = 0; it < 8; it++) {
            const int row = it * 4 + (lane >> 4), m = mblock + row;
            f32x4_t v = *(const f32x4_t *)(panel + row * PANEL_LD + c4);
            if (m < p.M) *(f32x4_t *)(out + (size_t)m * NP) = v;
        }
    }
}

template <int BM, int EPI>
int launch_bm(const MidParams &p, hipStream_t st) {
    static bool attr_set = false;
    const size_t lds = 2 * (size_t)(BM * BK * 2 + W_BYTES);
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)gemm_mid_kernel<BM, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) {
            vla_set_error("hipFuncSetAttribute(gemm_mid) failed: %s", hipGetErrorString(e));
            return VLA_EHIP;
        }
        attr_set = true;
    }
    gemm_mid_kernel<BM, EPI><<<p.n_tiles * p.splits, 256, lds, st>>>(p);
    return vla_check_launch("gemm_mid");
}

template <int EPI>
int launch_epi(const MidParams &p, hipStream_t st) {
    return p.M <= 128 ? launch_bm<128, EPI>(p, st) : launch_bm<256, EPI>(p, st);
}

}  // namespace

// Handles bf16 problems with M <= 256 (activation buffer readable up to 128 resp. 256 rows), K a multiple
// of 64 and weight segments that are multiples of 64 rows (SwiGLU: 32).  `scratch` holds the partial
// sums.  Returns 1 if handled, 0 if declined, < 0 on a launch error.
int try_gemm_bf16_mid(const GemmArgs &g, void *scratch, size_t scratch_bytes, hipStream_t st) {
    if (g.kblocked || g.M < 1 || g.M > 256 || g.K % BK != 0 || !scratch || g.epilogue == EPI_QKV_ROPE) return 0;
    const int bm = g.M <= 128 ? 128 : 256;
    if (g.a_rows < bm) return 0;
    MidParams p{};
    p.A = (const bf16_t *)g.A;
    p.W0 = (const bf16_t *)g.W[0]; p.W1 = (const bf16_t *)g.W[1]; p.W2 = (const bf16_t *)g.W[2];
    p.P = (float *)scratch; p.M = g.M; p.K = g.K; p.segN = g.segN;
    int np;
    if (g.epilogue == EPI_SWIGLU) {
        if (g.segN % 32 != 0) return 0;
        p.N = g.segN; p.n_tiles = g.segN / 32; np = 2 * p.N;
    } else {
        if (g.segN % BN != 0) return 0;
        p.N = g.n_seg * g.segN; p.n_tiles = p.N / BN; np = p.N;
    }
    const int ktiles = g.K / BK;
    // about two workgroups per CU, at least eight K tiles each, partial sums within the scratch buffer
    int splits = (512 + p.n_tiles - 1) / p.n_tiles;
    if (splits > ktiles / 8) splits = ktiles / 8;
    if (splits > 8) splits = 8;
    while (splits > 1 && (size_t)splits * g.M * np * sizeof(float) > scratch_bytes) splits--;
    if (splits < 1) splits = 1;
    if ((size_t)splits * g.M * np * sizeof(float) > scratch_bytes) return 0;
    p.splits = splits;
    const double flops = 2.0 * g.M * g.K * (double)np;
    int rc;
    {
        ProfScope ps(g.epilogue == EPI_SWIGLU ? "gemm_mid<swiglu>" : g.epilogue == EPI_RESIDUAL ? "gemm_mid<residual>" : "gemm_mid<store>", flops, st);
        if (g.epilogue == EPI_SWIGLU) rc = launch_epi<EPI_SWIGLU>(p, st);
        else rc = launch_epi<EPI_STORE>(p, st);         // store and residual differ only in the reduction
        if (rc) return rc;
    }
    if (g.deferred_splits && (g.epilogue == EPI_STORE || g.epilogue == EPI_RESIDUAL)) *g.deferred_splits = splits;
    else if ((rc = launch_splitk_reduce(g.epilogue, g.C, p.P, splits, g.M, p.N, st))) return rc;
    return 1;
}
