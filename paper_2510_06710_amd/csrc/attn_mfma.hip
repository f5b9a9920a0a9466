// Multi-row attention on MFMA for prefill, recompute and the parallel action-chunk pass
// (bf16, head_dim 64 or 128).  Rows at positions >= full_from see every key, rows below are causal.
//
// One wave owns 32 consecutive query rows of one (sequence, head) pair and walks the keys in blocks
// of 32 with an online softmax.  Both products run transposed so that no operand ever needs a
// cross-lane transpose:
//   S^T = K . Q^T   (MFMA rows = keys, columns = queries; K is stored [d/8][position][8], which is
//                    exactly the 16-byte (key, 8 dims) unit the row operand wants);
//   O^T = V^T . P^T (rows = head dims, columns = queries; the accumulator layout of S^T -- a lane
//                    holds one query column and 16 keys -- is directly the column operand P^T once
//                    the MFMA's k slots are assigned to those 16 keys; V^T comes from a transposed,
//                    blocked copy of V written by a small kernel beforehand).
// A lane therefore owns a single query for the whole kernel: running max, sum and the rescale of
// O^T are per-lane scalars, with one lane-xor-32 exchange per key block.
#include "vla_internal.h"

#include <type_traits>

namespace {

// V [position][d] of the cache -> VT [d/32][ps_pad/4][32][4]: for a block of 32 head dims, the four
// consecutive keys a lane needs are 8 contiguous bytes and the 32 lanes of a half-wave (32 dims) read
// 256 contiguous bytes.  Positions >= nk are written as zeros.
template <int D>
__global__ void __launch_bounds__(256) v_transpose_kernel(bf16_t *vt, const bf16_t *vc, int nk, int pos_stride,
                                                         int ps_pad) {
    __shared__ bf16_t tile[32][D + 8];
    const int item = blockIdx.y, kb = blockIdx.x;          // (sequence, head), key block of 32
    const bf16_t *vh = vc + (size_t)item * pos_stride * D;
    bf16_t *vth = vt + (size_t)item * D * ps_pad;
    for (int q = threadIdx.x; q < 32 * (D / 8); q += 256) {
        int r = q / (D / 8), c = q % (D / 8);
        int pos = kb * 32 + r;
        bf16x8_t v;
#pragma unroll
        for (int e = 0; e < 8; e++) v[e] = (bf16_t)0.f;
        if (pos < nk) v = *(const bf16x8_t *)(vh + (size_t)pos * D + c * 8);
#pragma unroll
        for (int e = 0; e < 8; e++) tile[r][c * 8 + e] = v[e];
    }
    __syncthreads();
    const int groups = ps_pad >> 2;
    for (int q = threadIdx.x; q < D * 8; q += 256) {        // (dim block, key group of this block, dim)
        int c = q & 31, g = (q >> 5) & 7, b = q >> 8;
        bf16x4_t v;
#pragma unroll
        for (int e = 0; e < 4; e++) v[e] = tile[g * 4 + e][b * 32 + c];
        *(bf16x4_t *)(vth + (((size_t)b * groups + kb * 8 + g) * 32 + c) * 4) = v;
    }
}

template <int D>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 4))) attn_prefill_kernel(bf16_t *out, const bf16_t *qbuf, const bf16_t *kc,
                                                          const bf16_t *vt, int R, int pos0, int full_from,
                                                          int n_heads, int pos_stride, int ps_pad, int H,
                                                          int q_blocks, int out_kb_rows) {
    constexpr int KS = D / 16;     // k steps of the S^T product
    constexpr int DB = D / 32;     // 32-row blocks of O^T
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int qb = blockIdx.x * 4 + wave;
    if (qb >= q_blocks) return;
    const int item = blockIdx.y;                       // sequence * n_heads + head
    const int s = item / n_heads, h = item - s * n_heads;
    const int nk = pos0 + R;
    const int col = lane & 31, hh = lane >> 5;
    const int r = min(qb * 32 + col, R - 1);           // this lane's query row (clamped; masked at store)
    const int qpos = pos0 + r;
    const int limit = (qpos >= full_from) ? nk : qpos + 1;     // keys [0, limit) are visible
    // largest limit in the wave decides how many key blocks to walk
    int wlimit = limit;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) wlimit = max(wlimit, __shfl_xor(wlimit, o, 64));
    const int n_kb = (wlimit + 31) >> 5;

    const bf16_t *qrow = qbuf + ((size_t)s * R + r) * H + (size_t)h * D;
    bf16x8_t qf[KS];
#pragma unroll
    for (int kk = 0; kk < KS; kk++) qf[kk] = *(const bf16x8_t *)(qrow + kk * 16 + hh * 8);

    const bf16_t *kh = kc + (size_t)item * D * pos_stride;
    const bf16_t *vth = vt + (size_t)item * D * ps_pad;
    const float scale = 1.0f / sqrtf((float)D);

    f32x16_t o_acc[DB];
#pragma unroll
    for (int b = 0; b < DB; b++)
#pragma unroll
        for (int i = 0; i < 16; i++) o_acc[b][i] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    // K fragments of key block kb (clamped key index: positions >= nk are masked below)
    auto load_k = [&](bf16x8_t (&kf)[KS], int kb) {
        const int key_ld = min(kb * 32 + col, nk - 1);
#pragma unroll
        for (int kk = 0; kk < KS; kk++)
            kf[kk] = *(const bf16x8_t *)(kh + ((size_t)(kk * 2 + hh) * pos_stride + key_ld) * 8);
    };
    bf16x8_t kf[KS], kf_next[KS];
    load_k(kf, 0);
    for (int kb = 0; kb < n_kb; kb++) {
        // ---- issue this block's V^T loads and the next block's K loads before any arithmetic ------------
        bf16x4_t vlo[2][DB], vhi[2][DB];
#pragma unroll
        for (int u = 0; u < 2; u++) {
            const int g0 = kb * 8 + 4 * u + hh;            // key group (4 keys) of slots e = 0..3
#pragma unroll
            for (int b = 0; b < DB; b++) {
                const bf16_t *vrow = vth + (((size_t)b * (ps_pad >> 2) + g0) * 32 + col) * 4;
                vlo[u][b] = *(const bf16x4_t *)vrow;
                vhi[u][b] = *(const bf16x4_t *)(vrow + 2 * 32 * 4);       // two key groups further
            }
        }
        load_k(kf_next, min(kb + 1, n_kb - 1));
        // ---- S^T block: rows = keys kb*32 .. +31, columns = the wave's 32 queries ---------------
        f32x16_t st;
#pragma unroll
        for (int i = 0; i < 16; i++) st[i] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KS; kk++) st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf[kk], st, 0, 0, 0);
        // register i of this lane is key kb*32 + 8*(i/4) + 4*hh + i%4 for query `col`
        float bmax = -INFINITY;
#pragma unroll
        for (int i = 0; i < 16; i++) {
            int key = kb * 32 + 8 * (i >> 2) + 4 * hh + (i & 3);
            float v = (key < limit) ? st[i] * scale : -INFINITY;
            st[i] = v;
            bmax = fmaxf(bmax, v);
        }
        bmax = fmaxf(bmax, __shfl_xor(bmax, 32, 64));
        const float m_new = fmaxf(m_run, bmax);
        // every query sees key 0, so after block 0 m_new is finite
        const float corr = __expf(m_run - m_new);
        // p is split into a bf16 head and a bf16 tail (two products below), so the probabilities
        // enter P.V with ~16 significant bits instead of 8
        float psum = 0.f;
        bf16x8_t pf[2], pl[2];
#pragma unroll
        for (int i = 0; i < 16; i++) {
            float p = __expf(st[i] - m_new);
            psum += p;
            bf16_t ph = (bf16_t)p;
            pf[i >> 3][i & 7] = ph;
            pl[i >> 3][i & 7] = (bf16_t)(p - (float)ph);
        }
        psum += __shfl_xor(psum, 32, 64);
        l_run = l_run * corr + psum;
        m_run = m_new;
        if (!__all(corr == 1.0f)) {                        // the running max moved for some query of the wave
#pragma unroll
            for (int b = 0; b < DB; b++)
#pragma unroll
                for (int i = 0; i < 16; i++) o_acc[b][i] *= corr;
        }
        // ---- O^T += V^T . P^T: k slot (hh, e) of product u is key kb*32 + 16u + 8*(e/4) + 4hh + e%4
#pragma unroll
        for (int u = 0; u < 2; u++) {
#pragma unroll
            for (int b = 0; b < DB; b++) {
                bf16x8_t vf;
#pragma unroll
                for (int e = 0; e < 4; e++) { vf[e] = vlo[u][b][e]; vf[4 + e] = vhi[u][b][e]; }
                o_acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[u], o_acc[b], 0, 0, 0);
                o_acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pl[u], o_acc[b], 0, 0, 0);
            }
        }
#pragma unroll
        for (int kk = 0; kk < KS; kk++) kf[kk] = kf_next[kk];
    }
    // ---- store: lane holds query `col`, dims b*32 + 8*(i/4) + 4*hh + i%4 -------------------------
    if (qb * 32 + col < R) {
        const float inv = 1.0f / l_run;
        // row-major [M, H], or the GEMM's k-blocked operand layout [H / 32][out_kb_rows][32]
        const size_t m = (size_t)s * R + r;
        bf16_t *orow = out_kb_rows ? out + ((size_t)h * (D / 32) * out_kb_rows + m) * 32 : out + m * H + (size_t)h * D;
        const size_t bstride = out_kb_rows ? (size_t)out_kb_rows * 32 : 32;
#pragma unroll
        for (int b = 0; b < DB; b++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
                bf16x4_t o;
#pragma unroll
                for (int e = 0; e < 4; e++) o[e] = (bf16_t)(o_acc[b][g * 4 + e] * inv);
                *(bf16x4_t *)(orow + b * bstride + g * 8 + 4 * hh) = o;
            }
    }
}

// ---- shared-key variant (head_dim 128) -------------------------------------------------------------------
// One workgroup owns NW consecutive 32-query blocks of one (sequence, head) pair, one wave per block, and walks
// the keys in blocks of 32 in lockstep: a key block is fetched once per workgroup into LDS (K as it is stored,
// V transposed on the way in) instead of once per wave from L2, which is what bounded the kernel above, and no
// transposed copy of V is needed in memory.  The arithmetic per wave is the same (same MFMA operand roles, same
// split of the probabilities into two bf16 terms).
//
// The fetching is the job of one extra wave: it holds no queries and no accumulators, so its registers take two
// whole key blocks (16 KB each), and the query waves need no staging registers at all.  In step kb it issues the
// loads of block kb + 2 into the register set that block kb held and writes block kb + 1 from the other set to
// LDS stage (kb + 1) % 2 while the query waves work on stage kb % 2; one barrier per step.
//
// LDS per stage: K  [16 dim chunks][32 keys][8]            8 KB, read back as 16-byte row operands;
//                VT [4 groups of 8 key slots][128 dims (+ one 16-byte pad per 8 dims)][8 slots]   9 KB; key
//                   16u + 8a + 4h + c (a, h in {0,1}, c < 4) sits in slot 16u + 8h + 4a + c, so that the eight keys
//                   a lane feeds to k slots (h, 0..7) of product u are the 16-byte unit (group 2u + h, its dim).
//                   Eight lanes = eight consecutive dims read 128 contiguous bytes: no bank conflicts.  The
//                   loading wave writes 4 bytes (a key pair of one dim) per lane, sixteen lanes eight dims apart:
//                   the pad puts those 144 instead of 128 bytes apart, a 2-way conflict instead of a 16-way one.
constexpr int ATT_K_BYTES = 16 * 32 * 16;
constexpr int ATT_VT_GROUP = 128 + 16;                 // 16-byte units per group of eight key slots: 128 dims + 1 pad per 8 dims
constexpr int ATT_VT_BYTES = 4 * ATT_VT_GROUP * 16;
constexpr int ATT_STAGE = ATT_K_BYTES + ATT_VT_BYTES;

template <int NW>
__global__ void __launch_bounds__((NW + 1) * 64) __attribute__((amdgpu_waves_per_eu(NW == 3 ? 3 : 1)))
attn_prefill_loader_kernel(bf16_t *out, const bf16_t *qbuf, const bf16_t *kc,
                                                                     const bf16_t *vc, int R, int pos0, int full_from,
                                                                     int n_heads, int pos_stride, int H, int q_blocks,
                                                                     int out_kb_rows, int n_items, int n_groups, int n_wgs) {
    constexpr int D = 128, KS = D / 16, DB = D / 32;
    constexpr int K_UNITS = 8;                         // 16-byte units of a K block per lane of the loading wave
    constexpr int V_UNITS = 4;                         // (key pair, 8 dims) units of a V block per lane
    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * ATT_STAGE];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: the two roles below are exclusive code paths
    // A (sequence, head) item has n_groups groups of NW query blocks, counted from the last block down: group 0 sees
    // the most key blocks, and when the block count is not a multiple of NW the last group is a ragged one that holds
    // the first blocks, which see the fewest keys.  One workgroup per group, except that the ragged group rides
    // along with the full group before it (n_wgs = n_groups - 1; the two are taken one after the other): a
    // workgroup of its own that lasts one or two key blocks costs about as much slot time in launching as in work
    // (at 294 rows = 10 blocks: 0.91 -> 0.72 ms per launch of 8192 items; pairing long with short groups throughout
    // was also tried and is slower where nothing is ragged, 0.65 against 0.58 ms at 288 rows).
    // Workgroup ids are dealt round-robin to the eight XCDs.  With an odd n_wgs the plain order (workgroup of the
    // item fastest) gives every XCD the same mix; with an even one, workgroup j of every item would land on the
    // same few XCDs, so there the ids of one XCD, taken in order, walk (item, j) with j fastest.
    int item, wg_j;                                    // item = sequence * n_heads + head
    {
        const int w = blockIdx.x;
        const int remapped = (n_wgs & 1) ? 0 : (n_items & ~7) * n_wgs;
        if (w < remapped) {
            const int local = w >> 3, il = local / n_wgs;
            item = il * 8 + (w & 7);
            wg_j = local - il * n_wgs;
        } else {
            item = w / n_wgs;
            wg_j = w - item * n_wgs;
        }
    }
    const int second_grp = (n_wgs != n_groups && wg_j == n_wgs - 1) ? n_groups - 1 : -1;
    const int s = item / n_heads, h = item - s * n_heads;
    const int nk = pos0 + R;
    const int col = lane & 31, hh = lane >> 5;
    const bf16_t *kh = kc + (size_t)item * D * pos_stride;
    const bf16_t *vh = vc + (size_t)item * pos_stride * D;
    // visible keys grow with the row, so the last row of a wave / of a group gives the block counts
    auto limit_of_row = [&](int row) { int p = pos0 + row; return (p >= full_from) ? nk : p + 1; };
    // key blocks that group `grp` walks (its last query row sees the most keys)
    auto key_blocks_of_group = [&](int grp) {
        const int g_last = min((q_blocks - grp * NW) * 32, R) - 1;
        return (limit_of_row(g_last) + 31) >> 5;
    };
    // After the last key block of a group every wave has passed the barrier that follows it, so the next group's
    // block 0 can go into stage 0 at once.  The role test is the outermost branch: what either role keeps across
    // its groups (addresses, masks) stays in that role's registers.

    // ---- the loading wave: global -> registers -> LDS, two key blocks in flight ------------------------------
    if (wave == NW) {
        bf16x8_t kreg[2][K_UNITS], vreg[2][V_UNITS][2];
        auto fetch = [&](auto set_c, int kb) {
            constexpr int SET = decltype(set_c)::value;
#pragma unroll
            for (int u = 0; u < K_UNITS; u++) {
                int q = lane + u * 64;                     // (dim chunk, key)
                int c = q >> 5, key = min(kb * 32 + (q & 31), nk - 1);
                kreg[SET][u] = *(const bf16x8_t *)((const char *)kh + (unsigned)(c * pos_stride + key) * 16u);
            }
#pragma unroll
            for (int u = 0; u < V_UNITS; u++) {
                int q = lane + u * 64;                     // (key pair, dim chunk): 16 lanes cover one key pair's 128 dims
                int t = q >> 4, c = q & 15;
                int k0 = min(kb * 32 + 2 * t, nk - 1), k1 = min(kb * 32 + 2 * t + 1, nk - 1);
                vreg[SET][u][0] = *(const bf16x8_t *)((const char *)vh + (unsigned)(k0 * D + c * 8) * 2u);
                vreg[SET][u][1] = *(const bf16x8_t *)((const char *)vh + (unsigned)(k1 * D + c * 8) * 2u);
            }
        };
        auto stash = [&](auto set_c, int stage) {
            constexpr int SET = decltype(set_c)::value;
            unsigned char *kb_lds = lds + stage * ATT_STAGE, *vt_lds = kb_lds + ATT_K_BYTES;
#pragma unroll
            for (int u = 0; u < K_UNITS; u++) *(bf16x8_t *)(kb_lds + (lane + u * 64) * 16) = kreg[SET][u];
#pragma unroll
            for (int u = 0; u < V_UNITS; u++) {
                int q = lane + u * 64;
                int t = q >> 4, c = q & 15;
                // key 2t = 16u' + 8a + 4h' + c' with c' even: slot 16u' + 8h' + 4a + c'
                int slot = (t >> 3) * 16 + ((t >> 1) & 1) * 8 + ((t >> 2) & 1) * 4 + (t & 1) * 2;
#pragma unroll
                for (int e = 0; e < 8; e++) {
                    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
                    bf16x2_t pr;
                    pr[0] = vreg[SET][u][0][e];
                    pr[1] = vreg[SET][u][1][e];
                    *(bf16x2_t *)(vt_lds + ((slot >> 3) * ATT_VT_GROUP + c * 9 + e) * 16 + (slot & 7) * 2) = pr;
                }
            }
        };
        using SA = std::integral_constant<int, 0>;
        using SB = std::integral_constant<int, 1>;
        for (int part = 0; part < 2; part++) {
            const int grp = part ? second_grp : wg_j;
            if (grp < 0) break;
            const int n_kb = key_blocks_of_group(grp);
            // The first two blocks have the same addresses for both groups.  Hiding that from the compiler keeps it
            // from holding those addresses in registers across the whole loop (they would spill).
            int kb0 = 0;
            asm volatile("" : "+s"(kb0));
            fetch(SA{}, kb0);
            if (n_kb > 1) fetch(SB{}, kb0 + 1);
            stash(SA{}, 0);
            __syncthreads();                               // block 0 is in stage 0
            // iteration kb: the other waves work on stage kb % 2; this one fetches block kb + 2 into the register
            // set that block kb held and moves block kb + 1 from the other set into stage (kb + 1) % 2
            for (int kb = 0; kb < n_kb; kb += 2) {
                if (kb + 2 < n_kb) fetch(SA{}, kb + 2);
                if (kb + 1 < n_kb) stash(SB{}, (kb + 1) & 1);
                __syncthreads();
                if (kb + 1 >= n_kb) break;
                if (kb + 3 < n_kb) fetch(SB{}, kb + 3);
                if (kb + 2 < n_kb) stash(SA{}, kb & 1);
                __syncthreads();
            }
        }
        return;
    }

    // ---- the query waves --------------------------------------------------------------------------------------
    for (int part = 0; part < 2; part++) {
        const int grp = part ? second_grp : wg_j;
        if (grp < 0) break;
        const int n_kb = key_blocks_of_group(grp);
        const int qb0 = q_blocks - (grp + 1) * NW;
        const int qb = max(qb0 + wave, 0);
        const bool active = qb0 + wave >= 0;
        const int r = min(qb * 32 + col, R - 1);
        const int qpos = pos0 + r;
        const int limit = (qpos >= full_from) ? nk : qpos + 1;      // keys [0, limit) are visible to this lane
        const int w_last = min(qb * 32 + 31, R - 1), w_first = min(qb * 32, R - 1);
        const int my_nkb = active ? (limit_of_row(w_last) + 31) >> 5 : 0;
        const int my_full_kb = limit_of_row(w_first) >> 5;          // blocks below this need no mask

        bf16x8_t qf[KS];
        {
            const bf16_t *qrow = qbuf + ((size_t)s * R + r) * H + (size_t)h * D;
#pragma unroll
            for (int kk = 0; kk < KS; kk++) qf[kk] = *(const bf16x8_t *)(qrow + kk * 16 + hh * 8);
        }
        f32x16_t o_acc[DB];
#pragma unroll
        for (int b = 0; b < DB; b++)
#pragma unroll
            for (int i = 0; i < 16; i++) o_acc[b][i] = 0.f;
        float m_run = -INFINITY, l_run = 0.f;
        const float c2 = 1.4426950408889634f / sqrtf((float)D);    // logits scale folded into the base-2 exponent

        __syncthreads();                                   // block 0 is in stage 0
        // An empty statement that reads the query fragments: their loads are waited for here, once.  Otherwise the
        // waits the compiler places in the loop must allow for a fragment still in flight on entry, and on every
        // later pass those same waits drain the prefetch of the next key block.
#pragma unroll
        for (int kk = 0; kk < KS; kk++) asm volatile("" ::"v"(qf[kk]));
        for (int kb = 0; kb < n_kb; kb++) {
            if (kb < my_nkb) {
                const unsigned char *k_lds = lds + (kb & 1) * ATT_STAGE, *vt_lds = k_lds + ATT_K_BYTES;
                // ---- S^T block: rows = keys kb*32 .. +31, columns = the wave's 32 queries -------------------
                f32x16_t st;
#pragma unroll
                for (int i = 0; i < 16; i++) st[i] = 0.f;
#pragma unroll
                for (int kk = 0; kk < KS; kk++) {
                    bf16x8_t kf = *(const bf16x8_t *)(k_lds + ((kk * 2 + hh) * 32 + col) * 16);
                    st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], st, 0, 0, 0);
                }
                // register i of this lane is key kb*32 + 8*(i/4) + 4*hh + i%4 for query `col`
                if (kb >= my_full_kb) {
#pragma unroll
                    for (int i = 0; i < 16; i++) {
                        int key = kb * 32 + 8 * (i >> 2) + 4 * hh + (i & 3);
                        st[i] = (key < limit) ? st[i] : -INFINITY;
                    }
                }
                float bmax = st[0];
#pragma unroll
                for (int i = 1; i < 16; i++) bmax = fmaxf(bmax, st[i]);
                bmax = fmaxf(bmax, __shfl_xor(bmax, 32, 64));
                const float m_new = fmaxf(m_run, bmax);    // every query sees key 0: finite from block 0 on
                const float corr = __builtin_amdgcn_exp2f((m_run - m_new) * c2);
                const float mc = m_new * c2;
                float psum = 0.f;
                bf16x8_t pf[2], pl[2];                      // p = bf16 head + bf16 tail: ~16 significant bits into P.V
#pragma unroll
                for (int i = 0; i < 16; i++) {
                    float p = __builtin_amdgcn_exp2f(fmaf(st[i], c2, -mc));
                    psum += p;
                    bf16_t ph = (bf16_t)p;
                    pf[i >> 3][i & 7] = ph;
                    pl[i >> 3][i & 7] = (bf16_t)(p - (float)ph);
                }
                psum += __shfl_xor(psum, 32, 64);
                l_run = l_run * corr + psum;
                m_run = m_new;
                if (!__all(corr == 1.0f)) {
#pragma unroll
                    for (int b = 0; b < DB; b++)
#pragma unroll
                        for (int i = 0; i < 16; i++) o_acc[b][i] *= corr;
                }
                // ---- O^T += V^T . P^T: k slot (hh, e) of product u is key kb*32 + 16u + 8*(e/4) + 4hh + e%4 --
#pragma unroll
                for (int u = 0; u < 2; u++) {
#pragma unroll
                    for (int b = 0; b < DB; b++) {
                        bf16x8_t vf = *(const bf16x8_t *)(vt_lds + ((2 * u + hh) * ATT_VT_GROUP + (b * 32 + col) + ((b * 32 + col) >> 3)) * 16);
                        o_acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[u], o_acc[b], 0, 0, 0);
                        o_acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pl[u], o_acc[b], 0, 0, 0);
                    }
                }
            }
            __syncthreads();
        }
        // ---- store: lane holds query `col`, dims b*32 + 8*(i/4) + 4*hh + i%4 ---------------------------------
        if (active && qb * 32 + col < R) {
            const float inv = 1.0f / l_run;
            const size_t m = (size_t)s * R + r;
            bf16_t *orow = out_kb_rows ? out + ((size_t)h * (D / 32) * out_kb_rows + m) * 32 : out + m * H + (size_t)h * D;
            const size_t bstride = out_kb_rows ? (size_t)out_kb_rows * 32 : 32;
#pragma unroll
            for (int b = 0; b < DB; b++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    bf16x4_t o;
#pragma unroll
                    for (int e = 0; e < 4; e++) o[e] = (bf16_t)(o_acc[b][g * 4 + e] * inv);
                    *(bf16x4_t *)(orow + b * bstride + g * 8 + 4 * hh) = o;
                }
        }
    }
}

template <int NW>
int launch_loader(bf16_t *out, const bf16_t *q, const bf16_t *kc, const bf16_t *vc, const RowsArgs &ra, const KvView &kv,
                  int H, int q_blocks, int n_items, int out_kb_rows, hipStream_t st) {
    const int n_groups = (q_blocks + NW - 1) / NW;
    // a ragged last group shares the workgroup of the group before it; VLA_ATTN_PAIR = 0 gives it its own (read
    // at every call: the tests switch it)
    const char *pe = getenv("VLA_ATTN_PAIR");
    const bool merge = n_groups > 1 && q_blocks % NW != 0 && !(pe && atoi(pe) == 0);
    const int n_wgs = merge ? n_groups - 1 : n_groups;
    attn_prefill_loader_kernel<NW><<<dim3(n_wgs * n_items), (NW + 1) * 64, 0, st>>>(
        out, q, kc, vc, ra.R, ra.pos0, ra.full_from, kv.n_heads, kv.pos_stride, H, q_blocks, out_kb_rows, n_items, n_groups,
        n_wgs);
    return vla_check_launch("attn_prefill");
}

inline int round_up32(int v) { return (v + 31) & ~31; }

}  // namespace

size_t attention_prefill_scratch_bytes(int n_seq, int n_heads, int d, int n_keys) {
    if (d != 64 && d != 128) return 0;
    return (size_t)n_seq * n_heads * d * round_up32(n_keys) * sizeof(bf16_t);
}

int try_attention_prefill_bf16(bf16_t *out, const bf16_t *q, const KvView &kv, int layer, const RowsArgs &ra,
                               int H, void *vt_scratch, int out_kb_rows, hipStream_t st) {
    if ((kv.d != 64 && kv.d != 128) || !vt_scratch || ra.R < 2) return 0;
    const int nk = ra.pos0 + ra.R, ps_pad = round_up32(nk);
    const int n_items = ra.n_seq * kv.n_heads;
    if (n_items == 0) return 1;
    if (n_items > 65535) return 0;                    // grid.y limit; the generic kernel takes over
    const bf16_t *kc = (const bf16_t *)kv.k + (size_t)layer * kv.layer_elems;
    const bf16_t *vc = (const bf16_t *)kv.v + (size_t)layer * kv.layer_elems;
    bf16_t *vt = (bf16_t *)vt_scratch;
    const int q_blocks = (ra.R + 31) / 32;
    int rc;
    auto pair_count = [&]() {                         // (query, visible key) pairs of one (sequence, head)
        double pairs = 0;
        for (int r = 0; r < ra.R; r++) pairs += (ra.pos0 + r >= ra.full_from) ? nk : ra.pos0 + r + 1;
        return pairs;
    };
    if (kv.d == 128) {
        ProfScope ps("attn_prefill", 4.0 * kv.d * pair_count() * n_items, st);
        // One wave per 32-query block, at most three of them plus the loading wave per workgroup: three such
        // workgroups fit a CU (35 KB LDS, 159 registers), each with two key blocks in flight.  Larger workgroups
        // fetch every key block fewer times but leave fewer independent workgroups per CU to cover the dependent
        // chain of a step (QK, softmax, PV); measured per 7B prefill step at 256 x 288 rows, with every wave also
        // loading: nine waves 26.0 ms, five or six 36-37 ms, four 21.6 ms; three + loading wave 19.9 ms (18.1 ms
        // with the padded V^T staging layout).
        switch (q_blocks <= 2 ? q_blocks : 3) {
        case 1: rc = launch_loader<1>(out, q, kc, vc, ra, kv, H, q_blocks, n_items, out_kb_rows, st); break;
        case 2: rc = launch_loader<2>(out, q, kc, vc, ra, kv, H, q_blocks, n_items, out_kb_rows, st); break;
        default: rc = launch_loader<3>(out, q, kc, vc, ra, kv, H, q_blocks, n_items, out_kb_rows, st); break;
        }
        return rc ? rc : 1;
    }
    {
        ProfScope ps("v_transpose", 2.0 * n_items * (double)nk * kv.d * 2.0, st);
        dim3 grid(ps_pad / 32, n_items);
        v_transpose_kernel<64><<<grid, 256, 0, st>>>(vt, vc, nk, kv.pos_stride, ps_pad);        // (head_dim 64 from here on)
        if ((rc = vla_check_launch("v_transpose"))) return rc;
    }
    {
        // algorithmic flops: 4 * d per (query, visible key) pair
        ProfScope ps("attn_prefill", 4.0 * kv.d * pair_count() * n_items, st);
        dim3 grid((q_blocks + 3) / 4, n_items);
        attn_prefill_kernel<64><<<grid, 256, 0, st>>>(out, q, kc, vt, ra.R, ra.pos0, ra.full_from, kv.n_heads,
                                                         kv.pos_stride, ps_pad, H, q_blocks, out_kb_rows);
        if ((rc = vla_check_launch("attn_prefill"))) return rc;
    }
    return 1;
}
