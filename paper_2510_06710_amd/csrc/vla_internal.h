// Internal declarations shared by the translation units of libvla (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "../../include/vla.h"

typedef __bf16 bf16_t;
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

#define VLA_WAVE 64

// ------------------------------------------------------------------------------------------
// KV buffer view.  One layer of K is [n_seq][n_heads][d/8][pos_stride][8] (eight consecutive
// head dims of one position are contiguous: the 16-byte unit both the streaming decode kernel
// and the MFMA operand loads want); one layer of V is [n_seq][n_heads][pos_stride][d].
// ------------------------------------------------------------------------------------------
struct KvView {
    void *k, *v;            // base of layer 0
    size_t layer_elems;     // elements per layer (same for K and V)
    int n_seq, n_heads, d, pos_stride;
};

struct RowsArgs {           // one forward over n_seq sequences x R new rows each
    int n_seq, R, pos0;     // row r of a sequence sits at absolute position pos0 + r
    int full_from;          // rows at positions >= full_from attend to all pos0 + R keys,
                            // rows below attend causally (keys 0..position)
};

enum GemmEpilogue { EPI_STORE = 0, EPI_RESIDUAL = 1, EPI_SWIGLU = 2, EPI_QKV_ROPE = 3 };

// Extra arguments of EPI_QKV_ROPE: the QKV projection whose epilogue rotates q and k and writes q to
// q_out [M, H] and k, v straight into layer `layer` of the KV buffer (head_dim 128 only).
struct QkvRopeArgs {
    void *q_out;            // may be NULL when the projection has no q segment (n_seg = 2: k and v only)
    const float2 *table;    // [R][d/2] (cos, sin)
    const KvView *kv;
    int layer;
    const RowsArgs *rows;
};

// k-blocked layouts ([K / 32][rows][32]) pad the row count of a block by this much, so that the 32-column blocks
// of one row panel do not sit an exact power-of-two distance apart.  (A precaution only: the L2's fetch traffic of
// the k-blocked GEMM, 2.3 times that of the row-major one, was the same with and without the pad, and also with a
// pad chosen to spread consecutive blocks over distinct sets of a modulo-indexed 4 MB cache.)
constexpr int VLA_KB_PAD_ROWS = 32;

struct GemmArgs {
    const void *A;          // [M, K] row-major (lda = K), storage dtype (or fp32 for fp32 models)
    const void *W[3];       // up to three weight segments, each [segN, K] row-major
    const void *Wkb[3];     // the same segments repacked k-blocked ([K / 32][segN + pad][32]) or NULL: kernels that stream
                            // the weights from HBM with row-major activations (decode forwards) prefer these
    int n_seg, segN;        // N = n_seg * segN (EPI_SWIGLU: W[0] = gate, W[1] = up, N = segN)
    void *C;                // EPI_STORE: fp32 [M, N]; EPI_SWIGLU: storage dtype [M, N]; EPI_RESIDUAL: fp32 [M, N] +=
    int M, K;
    int epilogue;
    const QkvRopeArgs *rope;   // EPI_QKV_ROPE only
    int kblocked;           // A (a_rows rows per 32-column block), the weights (segN rows per block, each segment
                            // on its own) and a SwiGLU output are stored [K / 32][rows][32]: direct-to-LDS kernel only
    int a_rows;             // rows of A that may be read (>= M; contents past M arbitrary): the MFMA kernel
                            // loads whole 256-row tiles and declines if the buffer does not cover them
    int *deferred_splits;   // not NULL (EPI_STORE and EPI_RESIDUAL of the split-K kernels): the kernel leaves its n
                            // partial products [n][M][N] at the start of the scratch buffer, puts n here and does not
                            // reduce them (the caller's next kernel adds them in order); 0 here: C is complete
    void *split_scratch;    // not NULL (EPI_STORE, row-major bf16): device scratch of split_scratch_bytes through which a
    size_t split_scratch_bytes;   // multi-row problem with few output tiles may cut its K range into parts
};

// ---- generic (any shape, fp32 or bf16 storage) kernels: kernels_generic.hip -----------------
template <typename T>
int launch_embed_prefix(float *X, const T *patch, const int32_t *ids, const T *embed, int n_seq, int P,
                        int T_, int row_stride_rows, int H, int vocab, hipStream_t st);
template <typename T>
int launch_embed_tokens(float *X, const int32_t *bins, int bins_stride, int n_tok, const T *embed,
                        int n_seq, int rows_per_seq, int row0, int H, int vocab, hipStream_t st);
template <typename T>
int launch_embed_slots(float *X, const T *slot_embed, int n_seq, int A, int rows_per_seq, int row0,
                       int H, hipStream_t st);
template <typename T>
int launch_rmsnorm(T *out, const float *X, const float *gain, int M, int H, float eps, hipStream_t st);
int launch_final_norm_rows(float *out, const float *X, const float *gain, int n_seq, int rows_per_seq,
                           int row0, int n_rows, int H, float eps, hipStream_t st);
template <typename T>
int launch_gemm_generic(const GemmArgs &g, hipStream_t st);
int launch_rope_table(float2 *table, int R, int pos0, int d, float theta, hipStream_t st);
// qkv is the fp32 [M, 3H] output of the QKV projection (never rounded before the rotation); the
// rotated q goes to q_out [M, H] in the storage dtype, k and v to the KV layout.
template <typename T>
int launch_rope_kv_write(T *q_out, const float *qkv, const float2 *table, const KvView &kv, int layer,
                         const RowsArgs &ra, int H, hipStream_t st);
template <typename T>
int launch_attention_generic(T *out, const T *q, const KvView &kv, int layer, const RowsArgs &ra,
                             int H, hipStream_t st);
// rows first .. first + count - 1 of each of n_seq sequences of R rows, packed
int launch_gather_rows(float *Xt, const float *X, int n_seq, int R, int first, int count, int H, hipStream_t st);
// rotary on q alone: qf fp32 [n_seq * count, H]; packed row m sits at table row first + m % count
template <typename T>
int launch_rope_q(T *q_out, const float *qf, const float2 *table, int n_seq, int count, int first, int n_heads, int d, int H,
                  hipStream_t st);
// Row i of h produces output index o = i * out_stride + out_off: bins_out[o], logp[o], ent[o],
// logits[o * 256 ..]; it reads gumbel[o * 256 ..] (if any) and given_bins[o] (if any: then the
// log-prob is that of the given bin and nothing is sampled).  If X_next is not NULL the embedding
// of token vocab - 256 + bin is written to X_next[i * H ..] as fp32.
template <typename T>
int launch_head_sample(const float *h, const T *lm_head_bins, int n_rows, int H, float temperature,
                       const float *gumbel, const int32_t *given_bins, int32_t *bins_out, float *logp,
                       float *ent, float *logits, int out_stride, int out_off, float *X_next,
                       const T *embed, int vocab, hipStream_t st);
int launch_value_head(float *value, const float *h, const float *w, float b, const float *bias, int vd, int n,
                      int H, int h_stride, hipStream_t st);

// silu(gate) * up of the bf16 fast paths: hardware exponential and reciprocal (1 ulp each, far below
// the bf16 rounding that follows); one formula for the prefill and the decode GEMMs so that both
// round the same way.
__device__ __forceinline__ float vla_silu_mul(float gate, float up) {
    return gate * __builtin_amdgcn_rcpf(1.0f + __expf(-gate)) * up;
}

// Maps a linear work-item id of the large-tile GEMMs to an output tile.  Workgroups are dealt round-robin to
// the eight XCDs, each with its own L2.  The ids of XCD y, taken in order, walk the tile rows y, y + 8, y + 16, ...
// in column panels of `GROUP` of those rows, so that the ~32 tiles resident on an XCD (4 x 8) share activation and
// weight rows in its L2 -- and all eight XCDs start at tile column 0 and move through the columns together, so
// that a weight panel that one XCD pulls from memory is found in the memory-side cache by the other seven
// (contiguous ranges of rows per XCD do the same only when the tile count per XCD is a whole number of panels).
// The row sets differ by one row at most while the ids are dealt evenly: an XCD that is through with its own rows
// takes, at the end, the tiles that the other XCDs' shares of ids do not reach.
// The arithmetic is the same in every lane; the results go back to scalar registers so that everything derived
// from them (tile base addresses) stays scalar.
__device__ __forceinline__ void vla_tile_of_block(int pid, int tiles_m, int tiles_n, int &tm, int &tn, int GROUP = 4) {
    const int total = tiles_m * tiles_n;
    const int q = total >> 3, r = total & 7;                 // XCDs below r are dealt q + 1 ids, the others q
    const int rows_lo = tiles_m >> 3, extra = tiles_m & 7;   // XCDs below `extra` own rows_lo + 1 tile rows
    auto ids_of = [&](int z) { return q + (z < r ? 1 : 0); };
    auto tiles_of = [&](int z) { return (rows_lo + (z < extra ? 1 : 0)) * tiles_n; };
    const int xcd = pid & 7, local = pid >> 3;
    int y = xcd, l = local;                                  // tile l of XCD y's own rows
    if (local >= tiles_of(xcd)) {
        int e = local - tiles_of(xcd);                       // index into the tiles left over, pooled in XCD order
        for (int z = 0; z < 8; z++)
            if (z < xcd) e += max(ids_of(z) - tiles_of(z), 0);
        for (int z = 0; z < 8; z++) {
            const int left = tiles_of(z) - ids_of(z);
            if (left > 0) {
                if (e < left) { y = z; l = ids_of(z) + e; break; }
                e -= left;
            }
        }
    }
    const int rows_y = rows_lo + (y < extra ? 1 : 0);
    // GROUP = 4: measured best of 1, 2, 4, 6, 8, 16, 32 on the 7B shapes (the QKV projection passes 2)
    const int panel = l / (GROUP * tiles_n);
    const int first = panel * GROUP;
    const int rows = min(GROUP, rows_y - first);
    const int in_panel = l - panel * GROUP * tiles_n;
    tm = __builtin_amdgcn_readfirstlane(y + 8 * (first + in_panel % rows));
    tn = __builtin_amdgcn_readfirstlane(in_panel / rows);
}

// ---- gfx950 fast paths (bf16, aligned shapes); each returns 1 if it handled the call, 0 if the
// shape is outside what it supports (caller then uses the generic kernel), <0 on launch error ----
int try_gemm_bf16_dma(const GemmArgs &g, hipStream_t st);
int try_gemm_bf16_dma_splitk(const GemmArgs &g, void *scratch, size_t scratch_bytes, hipStream_t st);
int try_gemm_bf16_dma_splitk_rows(const GemmArgs &g, void *scratch, size_t scratch_bytes, hipStream_t st);
int launch_weight_kblock(bf16_t *dst, const bf16_t *src, int N, int K, hipStream_t st);
// qkv: `splits` partial copies of the fp32 [M, 3H] projection, `split_stride` floats apart, added in order
int launch_rope_kv_write_bf16(bf16_t *q_out, const float *qkv, int splits, size_t split_stride, const float2 *table,
                              const KvView &kv, int layer, const RowsArgs &ra, int H, hipStream_t st);
// x[m] += sum of the `splits` partial rows P[k][m] (in order); then, if gain != NULL, out[m] = RMSNorm(x[m]) * gain as
// bf16, row-major.  Returns 1 if handled (H a multiple of 1024, at most 8192), 0 otherwise.
int try_reduce_residual_rmsnorm_bf16(bf16_t *out, float *X, const float *P, int splits, int M, int H, const float *gain,
                                     float eps, hipStream_t st);
// kb_rows = 0: row-major output [M, H]; else k-blocked [H / 32][kb_rows][32]
int try_rmsnorm_bf16(bf16_t *out, const float *X, const float *gain, int M, int H, float eps, int kb_rows, hipStream_t st);
int try_gemm_bf16_skinny(const GemmArgs &g, void *scratch, hipStream_t st);
int try_gemm_bf16_mid(const GemmArgs &g, void *scratch, size_t scratch_bytes, hipStream_t st);
int launch_splitk_reduce(int epilogue, void *C, const float *P, int splits, int M, int N, hipStream_t st);
size_t gemm_skinny_scratch_bytes(int M, int max_n);
// out_kb_rows = 0: row-major output [M, H]; else k-blocked [H / 32][out_kb_rows][32]
int try_attention_prefill_bf16(bf16_t *out, const bf16_t *q, const KvView &kv, int layer,
                               const RowsArgs &ra, int H, void *vt_scratch, int out_kb_rows, hipStream_t st);
int try_attention_decode_bf16(bf16_t *out, const bf16_t *q, const KvView &kv, int layer,
                              const RowsArgs &ra, int H, hipStream_t st);
size_t attention_prefill_scratch_bytes(int n_seq, int n_heads, int d, int n_keys);

int vla_check_launch(const char *what);
void vla_set_error(const char *fmt, ...);

// The host-side model object behind the opaque handle of the C ABI.
struct vla_model {
    vla_config cfg;
    vla_weights w;
    std::vector<vla_layer_weights> layers;
    std::vector<vla_layer_weights> packed;   // k-blocked copies of the seven projection matrices (vla_prepack), or empty
};
int vla_check_config(const vla_config *c);                                   // VLA_OK or the error code, message set
int vla_check_rows_per_pass(const vla_config &c, long n_seq, long rows_per_seq);
// C = A . W^T of a multi-row forward (row-major operands): the MFMA kernels where the shape allows, else the generic one
int vla_gemm_dispatch(const vla_config &c, const GemmArgs &g, hipStream_t st);
// The teacher-forced forward of the log-prob recompute over n rollouts (the kernels vla_logprob_recompute runs, every
// row through every layer), keeping the fp32 residual stream at the input of layer l in keep + l * n * R * H
// ([n * R, H] each).  *x_final: the residual stream after the last layer ([n * R, H], inside fw_ws).  fw_ws: device
// scratch of vla_forward_streams_bytes(c, n_max, R) bytes with n <= n_max.
size_t vla_forward_streams_bytes(const vla_config &c, int n_max, int R);
int vla_forward_streams(vla_model *m, void *fw_ws, int n_max, const void *patch, const int32_t *ids, const int32_t *bins, int n,
                        int P, int T, int A, int mode, const void *slot_embed, float *keep, const float **x_final, hipStream_t st);

// Profiling scope: when profiling is enabled, records an event pair around the launches issued
// during its lifetime, tagged with `label` (a string literal) and the algorithmic work.
struct ProfScope {
    ProfScope(const char *label, double work, hipStream_t st);
    ~ProfScope();
    int slot;
    hipStream_t st;
};
