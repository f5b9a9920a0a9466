// C-ABI entry points of libvla: argument validation, workspace planning and the host-side
// sequencing of kernels.  All arithmetic lives in the kernels; this file only enqueues them.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <new>
#include <vector>

#include "vla_internal.h"

// ------------------------------------------------------------------------------------------ errors
static thread_local char g_err[512] = "";

void vla_set_error(const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int vla_check_launch(const char *what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        vla_set_error("launch of %s failed: %s", what, hipGetErrorString(e));
        return VLA_EHIP;
    }
    return 0;
}


// ------------------------------------------------------------------------------------------ profiling
struct ProfRecord { const char *label; double work; hipEvent_t e0, e1; };
static bool g_prof_on = false;
static std::vector<ProfRecord> g_prof;          // records in use
static std::vector<hipEvent_t> g_event_pool;    // events kept for reuse

static hipEvent_t prof_event() {
    if (!g_event_pool.empty()) { hipEvent_t e = g_event_pool.back(); g_event_pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

ProfScope::ProfScope(const char *label, double work, hipStream_t s) : slot(-1), st(s) {
    if (!g_prof_on) return;
    ProfRecord r{label, work, prof_event(), prof_event()};
    if (!r.e0 || !r.e1) return;
    (void)hipEventRecord(r.e0, st);
    g_prof.push_back(r);
    slot = (int)g_prof.size() - 1;
}
ProfScope::~ProfScope() {
    if (slot >= 0) (void)hipEventRecord(g_prof[slot].e1, st);
}

static void prof_clear() {
    for (auto &r : g_prof) { g_event_pool.push_back(r.e0); g_event_pool.push_back(r.e1); }
    g_prof.clear();
}

// ------------------------------------------------------------------------------------------ config
static int check_config(const vla_config *c) {
    if (!c) { vla_set_error("config is NULL"); return VLA_EINVAL; }
    if (c->dtype != VLA_DTYPE_F32 && c->dtype != VLA_DTYPE_BF16) {
        vla_set_error("unknown dtype %d", c->dtype);
        return VLA_EDTYPE;
    }
    if (c->n_layers <= 0 || c->hidden <= 0 || c->n_heads <= 0 || c->ffn <= 0 || c->vocab <= 0 ||
        c->max_batch <= 0 || c->max_seq <= 0 || !(c->rms_eps > 0.f) || !(c->rope_theta > 0.f)) {
        vla_set_error("config has a non-positive size, eps or theta");
        return VLA_EINVAL;
    }
    if (c->n_bins != VLA_N_BINS) { vla_set_error("n_bins = %d unsupported (must be 256)", c->n_bins); return VLA_ESHAPE; }
    if (c->vocab < VLA_N_BINS) { vla_set_error("vocab %d smaller than the 256 action bins", c->vocab); return VLA_ESHAPE; }
    if (c->hidden % c->n_heads != 0) { vla_set_error("hidden %d not divisible by n_heads %d", c->hidden, c->n_heads); return VLA_ESHAPE; }
    int d = c->hidden / c->n_heads;
    if (d % 16 != 0 || d > 256) { vla_set_error("head_dim %d unsupported (multiple of 16, at most 256)", d); return VLA_ESHAPE; }
    if (c->max_seq > 8192) { vla_set_error("max_seq %d unsupported (at most 8192)", c->max_seq); return VLA_ESHAPE; }
    if (c->value_dim < 0 || c->value_dim > 1024) { vla_set_error("value_dim %d unsupported (0..1024)", c->value_dim); return VLA_ESHAPE; }
    if (c->hidden > 8192) { vla_set_error("hidden %d unsupported (at most 8192)", c->hidden); return VLA_ESHAPE; }
    return VLA_OK;
}

static inline int value_dim(const vla_config &c) { return c.value_dim > 0 ? c.value_dim : 1; }
static inline size_t elt_size(const vla_config &c) { return c.dtype == VLA_DTYPE_F32 ? 4 : 2; }
static inline size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

static size_t kv_layer_elems(const vla_config &c, int n_seq) {
    return (size_t)n_seq * c.hidden * c.max_seq;
}

// ------------------------------------------------------------------------------------------ workspace
struct Workspace {
    float *X;        // residual stream fp32 [M, H]
    void *Nrm;       // norm output, storage dtype [M, H]
    float *QKV;      // QKV projection, fp32 [M, 3H] (rounded only after the rotation)
    void *Q;         // rotated q, storage dtype [M, H]
    void *AO;        // attention output [M, H]
    void *ACT;       // SwiGLU output [M, F]
    float2 *rope;    // [R, d/2]
    float *Hb;       // final-norm rows fp32 [head_rows, H]
    void *kvs_k, *kvs_v;   // one-layer KV scratch (recompute)
    void *vt;        // scratch of the MFMA prefill attention
    void *skinny;    // split-K partial sums of the decode GEMM (single-row forwards only)
    int a_rows;      // rows allocated for Nrm, AO and ACT (M rounded up to whole 256-row GEMM tiles, plus the pad of
                     // the k-blocked layout, whose block stride this is)
    // Tail of the last layer (see run_layers): the rows whose output is read, packed [n_seq * tail_rows, ...]
    int tail_rows;   // rows per sequence (0: no tail buffers)
    float *tX, *tQf; // residual stream and fp32 q projection of the tail rows
    void *tNrm, *tQ, *tAO, *tACT, *tskinny;
    int t_a_rows;
    size_t total;
};

// Lays the workspace out from `base` (may be NULL to only size it).
static Workspace plan_workspace(const vla_config &c, char *base, int n_seq, int R, int n_keys,
                                int head_rows, bool kv_scratch, int tail_rows = 0) {
    Workspace w;
    size_t off = 0, es = elt_size(c);
    size_t M = (size_t)n_seq * R, H = c.hidden, F = c.ffn;
    auto take = [&](size_t bytes) { char *p = base ? base + off : nullptr; off += align_up(bytes); return (void *)p; };
    // GEMM activation operands are padded to whole tiles of 256 rows: the MFMA kernel reads (and
    // discards the products of) the rows between M and the end of its last tile
    size_t Mp = (M + 255) / 256 * 256 + VLA_KB_PAD_ROWS;
    w.a_rows = (int)Mp;
    w.X = (float *)take(M * H * 4);
    w.Nrm = take(Mp * H * es);
    w.QKV = (float *)take(M * 3 * H * 4);
    w.Q = take(M * H * es);
    w.AO = take(Mp * H * es);
    w.ACT = take(Mp * F * es);
    w.rope = (float2 *)take((size_t)R * (H / c.n_heads / 2) * sizeof(float2));
    w.Hb = (float *)take((size_t)head_rows * H * 4);
    w.kvs_k = kv_scratch ? take(kv_layer_elems(c, n_seq) * es) : nullptr;
    w.kvs_v = kv_scratch ? take(kv_layer_elems(c, n_seq) * es) : nullptr;
    size_t vtb = (c.dtype == VLA_DTYPE_BF16 && R > 1)
                     ? attention_prefill_scratch_bytes(n_seq, c.n_heads, c.hidden / c.n_heads, n_keys) : 0;
    w.vt = vtb ? take(vtb) : nullptr;
    size_t skb = (c.dtype == VLA_DTYPE_BF16 && R == 1 && M <= 256) ? gemm_skinny_scratch_bytes((int)M, (int)(2 * F > 3 * H ? 2 * F : 3 * H)) : 0;
    w.skinny = skb ? take(skb) : nullptr;
    w.tail_rows = tail_rows;
    w.tX = w.tQf = nullptr; w.tNrm = w.tQ = w.tAO = w.tACT = w.tskinny = nullptr; w.t_a_rows = 0;
    if (tail_rows > 0) {
        const size_t Mt = (size_t)n_seq * tail_rows, Mtp = (Mt + 255) / 256 * 256 + VLA_KB_PAD_ROWS;
        w.t_a_rows = (int)Mtp;
        w.tX = (float *)take(Mt * H * 4);
        w.tQf = (float *)take(Mt * H * 4);
        w.tNrm = take(Mtp * H * es);
        w.tQ = take(Mtp * H * es);
        w.tAO = take(Mtp * H * es);
        w.tACT = take(Mtp * F * es);
        const size_t tsk = (c.dtype == VLA_DTYPE_BF16 && Mt <= 256) ? gemm_skinny_scratch_bytes((int)Mt, (int)(2 * F > 3 * H ? 2 * F : 3 * H)) : 0;
        w.tskinny = tsk ? take(tsk) : nullptr;
    }
    w.total = off;
    return w;
}

// The kernels index a pass's activation buffers with 32-bit byte offsets: the residual stream ([rows, H] fp32) and
// the widest activation operand ([rows rounded up to tiles + pad, max(H, F)] in the storage dtype) must each stay
// below 2 GiB.  7B shape, bf16: 97,254 rows per pass (the benchmark's largest pass has 75,264).
static long max_rows_per_pass(const vla_config &c) {
    const long lim = 0x7fffffffL;
    long wide = c.ffn > c.hidden ? c.ffn : c.hidden;
    long by_x = lim / ((long)c.hidden * 4);
    long by_act = lim / (wide * (long)elt_size(c)) - 256 - VLA_KB_PAD_ROWS;
    return by_x < by_act ? by_x : by_act;
}

static int check_rows_per_pass(const vla_config &c, long n_seq, long rows_per_seq) {
    long lim = max_rows_per_pass(c);
    if (n_seq * rows_per_seq > lim) {
        vla_set_error("%ld sequences x %ld rows exceed the %ld rows one pass can hold at this shape: split the batch",
                      n_seq, rows_per_seq, lim);
        return VLA_ESHAPE;
    }
    return VLA_OK;
}

// rollouts per pass of the recompute: the capacity, cut down to what one pass can hold (at least 1).  R is S + A,
// the rows of the longer of the two modes, for either mode: the size query does not know the mode.
static int recompute_micro_batch(const vla_config &c, int N, int R) {
    long mb = N < c.max_batch ? N : c.max_batch;
    long fit = max_rows_per_pass(c) / (R > 0 ? R : 1);
    if (mb > fit) mb = fit;
    return mb > 0 ? (int)mb : 1;
}

// ------------------------------------------------------------------------------------------ forward
// Triage switch (vla_debug_force_generic): a bit mask that sends a step to the shape-generic kernel even when a
// gfx950 fast path applies (1 large GEMM, 2 decode GEMM, 4 multi-row attention, 8 decode attention, 16 rotary / KV
// write / RMSNorm).  Process-wide; 0 unless the caller sets it.
static int g_force_generic = 0;
static int force_generic() { return g_force_generic; }

// The multi-row bf16 forwards can run on k-blocked operands ([K / 32][rows][32], see gemm_dma.hip): needs
// head_dim 128 (fused rotation epilogue), tile-aligned widths and repacked weights.
static bool kblocked_shape_ok(const vla_config &c) {
    if (c.dtype != VLA_DTYPE_BF16 || c.hidden % c.n_heads != 0 || c.hidden / c.n_heads != 128) return false;
    if (c.hidden % 1024 != 0 || c.hidden > 8192) return false;        // the register-resident RMSNorm writes the layout
    return c.hidden % 256 == 0 && c.hidden >= 256 && c.ffn % 128 == 0 && c.ffn >= 256 &&
           (size_t)c.ffn * c.hidden * 2 < ((size_t)1 << 31);
}
static size_t prepack_layer_bytes(const vla_config &c) {
    const size_t H = c.hidden, F = c.ffn, P = VLA_KB_PAD_ROWS;                       // every matrix a multiple of 256 bytes
    return (4 * (H + P) * H + 2 * (F + P) * H + (H + P) * F) * 2;
}

// The large-tile GEMM (declines K below 256 or not a multiple of 64: the generic kernel then takes the call).
static int try_gemm_bf16_large(const GemmArgs &g, hipStream_t st) { return try_gemm_bf16_dma(g, st); }

// Kernel choice depends on the storage type, on whether the forward has one row per sequence (decode) and, for
// decode forwards, on the batch: up to 128 rows stream the weights through the skinny kernel, larger batches use
// the split-K tile kernels.  The K ranges, and with them the order in which a row's products are summed, therefore
// differ between batch sizes on either side of 128 (each configuration by itself is deterministic, and within one
// call a row's result does not depend on the other rows).
template <typename T>
static int run_gemm(const vla_config &c, GemmArgs g, void *skinny_scratch, hipStream_t st) {
    if (c.dtype == VLA_DTYPE_BF16) {
        int r = 0;
        if (skinny_scratch && !(force_generic() & 2)) {
            // single-row forwards: up to 128 rows stream the weights through the skinny kernel; above
            // that the work is MFMA bound and the large tile with split K does better
            if (g.M > 128 && !(force_generic() & 1)) {
                const size_t sb = gemm_skinny_scratch_bytes(g.M, 2 * c.ffn > 3 * c.hidden ? 2 * c.ffn : 3 * c.hidden);
                r = try_gemm_bf16_dma_splitk(g, skinny_scratch, sb, st);
                if (r == 0) r = try_gemm_bf16_mid(g, skinny_scratch, sb, st);
            }
            if (r == 0) r = try_gemm_bf16_skinny(g, skinny_scratch, st);
        }
        if (r != 0) return r < 0 ? r : 0;
        if (g.split_scratch && !(force_generic() & 1)) r = try_gemm_bf16_dma_splitk_rows(g, g.split_scratch, g.split_scratch_bytes, st);
        if (r != 0) return r < 0 ? r : 0;
        r = (force_generic() & 1) ? 0 : try_gemm_bf16_large(g, st);
        if (r != 0) return r < 0 ? r : 0;
    }
    return launch_gemm_generic<T>(g, st);
}

// All decoder layers over n_seq x R new rows held in ws.X; K, V of the new rows go to `kv`
// (layer l of it, or layer 0 when `kv` is a one-layer scratch).
template <typename T>
static int run_rmsnorm(const vla_config &c, void *out, const float *X, const void *gain, int M, int kb_rows,
                       hipStream_t st) {
    if (c.dtype == VLA_DTYPE_BF16 && !(force_generic() & 16)) {
        int r = try_rmsnorm_bf16((bf16_t *)out, X, (const float *)gain, M, c.hidden, c.rms_eps, kb_rows, st);
        if (r != 0) return r < 0 ? r : 0;
    }
    if (kb_rows) { vla_set_error("internal: k-blocked RMSNorm output unavailable for hidden %d", c.hidden); return VLA_ESHAPE; }
    return launch_rmsnorm<T>((T *)out, X, (const float *)gain, M, c.hidden, c.rms_eps, st);
}

// One decoder layer on k-blocked activations and repacked weights: every GEMM is the direct-to-LDS kernel,
// whose operands are then whole cache lines (multi-row bf16 forwards at head_dim 128 only).
static int run_layer_kblocked(const vla_model *m, const Workspace &ws, const RowsArgs &ra, const KvView &kv, int l, int kl,
                              hipStream_t st) {
    const vla_config &c = m->cfg;
    const int H = c.hidden, F = c.ffn, M = ra.n_seq * ra.R;
    const vla_layer_weights &lw = m->layers[l], &pk = m->packed[l];
    int rc;
    auto must = [&](int r, const char *what) {
        if (r == 0) { vla_set_error("internal: k-blocked path declined at %s", what); return (int)VLA_ESHAPE; }
        return r < 0 ? r : 0;
    };
    if ((rc = must(try_rmsnorm_bf16((bf16_t *)ws.Nrm, ws.X, (const float *)lw.attn_norm, M, H, c.rms_eps, ws.a_rows, st), "attn norm"))) return rc;
    QkvRopeArgs qa{ws.Q, ws.rope, &kv, kl, &ra};
    GemmArgs g{};
    g.A = ws.Nrm; g.W[0] = pk.wq; g.W[1] = pk.wk; g.W[2] = pk.wv; g.n_seg = 3; g.segN = H; g.C = nullptr; g.M = M; g.K = H;
    g.epilogue = EPI_QKV_ROPE; g.rope = &qa; g.a_rows = ws.a_rows; g.kblocked = 1;
    if ((rc = must(try_gemm_bf16_dma(g, st), "QKV projection"))) return rc;
    if ((rc = must(try_attention_prefill_bf16((bf16_t *)ws.AO, (const bf16_t *)ws.Q, kv, kl, ra, H, ws.vt, ws.a_rows, st), "attention"))) return rc;
    g = GemmArgs{};
    g.A = ws.AO; g.W[0] = pk.wo; g.n_seg = 1; g.segN = H; g.C = ws.X; g.M = M; g.K = H; g.epilogue = EPI_RESIDUAL;
    g.a_rows = ws.a_rows; g.kblocked = 1;
    if ((rc = must(try_gemm_bf16_dma(g, st), "O projection"))) return rc;
    if ((rc = must(try_rmsnorm_bf16((bf16_t *)ws.Nrm, ws.X, (const float *)lw.ffn_norm, M, H, c.rms_eps, ws.a_rows, st), "ffn norm"))) return rc;
    g = GemmArgs{};
    g.A = ws.Nrm; g.W[0] = pk.w_gate; g.W[1] = pk.w_up; g.n_seg = 2; g.segN = F; g.C = ws.ACT; g.M = M; g.K = H;
    g.epilogue = EPI_SWIGLU; g.a_rows = ws.a_rows; g.kblocked = 1;
    if ((rc = must(try_gemm_bf16_dma(g, st), "gate/up projection"))) return rc;
    g = GemmArgs{};
    g.A = ws.ACT; g.W[0] = pk.w_down; g.n_seg = 1; g.segN = H; g.C = ws.X; g.M = M; g.K = F; g.epilogue = EPI_RESIDUAL;
    g.a_rows = ws.a_rows; g.kblocked = 1;
    return must(try_gemm_bf16_dma(g, st), "down projection");
}

// The rows of a multi-row forward whose final hidden state is read: `count` rows per sequence from row `first`.
struct TailSpec { int first, count; };

// Whether a forward of R rows per sequence takes the shortened last layer.  Only the rows that the head (or the value
// head) reads need the last layer's attention output and feed-forward block; all rows still need its K and V, which
// the KV cache keeps.  So the last layer computes K and V for every row and everything else for the tail rows alone
// (packed), which leaves the outputs unchanged and saves (1 - 2H^2 / (4H^2 + 3HF)) of one layer's GEMMs: 2.6 % of a
// 32-layer prefill.  Not worth it when the tail is a large share of the rows.
static bool use_tail(const TailSpec *tail, int R) { return tail && tail->count >= 1 && tail->count * 4 <= R; }

// Last layer, tail form: K, V of all rows (ws.X / ws.Nrm as in any layer), then the rest of the layer on the packed
// tail rows (ws.tX and friends) with the kernels a forward of that many rows would use.
template <typename T>
static int run_last_layer_tail(const vla_model *m, const Workspace &ws, const RowsArgs &ra, const KvView &kv, int l, int kl,
                               const TailSpec &tail, bool kb, hipStream_t st) {
    const vla_config &c = m->cfg;
    const int H = c.hidden, F = c.ffn, M = ra.n_seq * ra.R, d = H / c.n_heads, Mt = ra.n_seq * tail.count;
    const vla_layer_weights &lw = m->layers[l];
    int rc;
    // ---- K and V of every row
    bool kv_done = false;
    if (c.dtype == VLA_DTYPE_BF16 && d == 128 && !(force_generic() & (1 | 16))) {
        QkvRopeArgs qa{nullptr, ws.rope, &kv, kl, &ra};
        GemmArgs g{};
        g.A = ws.Nrm; g.n_seg = 2; g.segN = H; g.C = nullptr; g.M = M; g.K = H; g.epilogue = EPI_QKV_ROPE; g.rope = &qa; g.a_rows = ws.a_rows;
        if (kb) {
            if ((rc = try_rmsnorm_bf16((bf16_t *)ws.Nrm, ws.X, (const float *)lw.attn_norm, M, H, c.rms_eps, ws.a_rows, st)) <= 0)
                return rc < 0 ? rc : (vla_set_error("internal: k-blocked RMSNorm declined"), (int)VLA_ESHAPE);
            g.W[0] = m->packed[l].wk; g.W[1] = m->packed[l].wv; g.kblocked = 1;
        } else {
            if ((rc = run_rmsnorm<T>(c, ws.Nrm, ws.X, lw.attn_norm, M, 0, st))) return rc;
            g.W[0] = lw.wk; g.W[1] = lw.wv;
        }
        rc = try_gemm_bf16_dma(g, st);
        if (rc < 0) return rc;
        if (rc == 0 && kb) { vla_set_error("internal: k-blocked K / V projection declined"); return VLA_ESHAPE; }
        kv_done = rc == 1;
    }
    if (!kv_done) {          // plain path: the full projection (its q rows are not used), rotation and KV write
        if ((rc = run_rmsnorm<T>(c, ws.Nrm, ws.X, lw.attn_norm, M, 0, st))) return rc;
        GemmArgs g{};
        g.A = ws.Nrm; g.W[0] = lw.wq; g.W[1] = lw.wk; g.W[2] = lw.wv; g.n_seg = 3; g.segN = H; g.C = ws.QKV; g.M = M; g.K = H;
        g.epilogue = EPI_STORE; g.a_rows = ws.a_rows;
        if ((rc = run_gemm<T>(c, g, nullptr, st))) return rc;
        if (c.dtype == VLA_DTYPE_BF16 && !(force_generic() & 16))
            rc = launch_rope_kv_write_bf16((bf16_t *)ws.Q, ws.QKV, 1, (size_t)M * 3 * H, ws.rope, kv, kl, ra, H, st);
        else rc = launch_rope_kv_write<T>((T *)ws.Q, ws.QKV, ws.rope, kv, kl, ra, H, st);
        if (rc) return rc;
    }
    // ---- the tail rows: q, attention against the layer's K and V, O projection, feed-forward block
    if ((rc = launch_gather_rows(ws.tX, ws.X, ra.n_seq, ra.R, tail.first, tail.count, H, st))) return rc;
    if ((rc = run_rmsnorm<T>(c, ws.tNrm, ws.tX, lw.attn_norm, Mt, 0, st))) return rc;
    GemmArgs g{};
    g.A = ws.tNrm; g.W[0] = lw.wq; g.n_seg = 1; g.segN = H; g.C = ws.tQf; g.M = Mt; g.K = H; g.epilogue = EPI_STORE; g.a_rows = ws.t_a_rows;
    if ((rc = run_gemm<T>(c, g, ws.tskinny, st))) return rc;
    if ((rc = launch_rope_q<T>((T *)ws.tQ, ws.tQf, ws.rope, ra.n_seq, tail.count, tail.first, c.n_heads, d, H, st))) return rc;
    const RowsArgs rt{ra.n_seq, tail.count, ra.pos0 + tail.first, ra.full_from};
    int done = 0;
    if (c.dtype == VLA_DTYPE_BF16) {
        if (tail.count == 1)
            done = (force_generic() & 8) ? 0 : try_attention_decode_bf16((bf16_t *)ws.tAO, (const bf16_t *)ws.tQ, kv, kl, rt, H, st);
        else
            done = (force_generic() & 4) ? 0 : try_attention_prefill_bf16((bf16_t *)ws.tAO, (const bf16_t *)ws.tQ, kv, kl, rt, H, ws.vt, 0, st);
        if (done < 0) return done;
    }
    if (!done && (rc = launch_attention_generic<T>((T *)ws.tAO, (const T *)ws.tQ, kv, kl, rt, H, st))) return rc;
    g = GemmArgs{};
    g.A = ws.tAO; g.W[0] = lw.wo; g.n_seg = 1; g.segN = H; g.C = ws.tX; g.M = Mt; g.K = H; g.epilogue = EPI_RESIDUAL; g.a_rows = ws.t_a_rows;
    if ((rc = run_gemm<T>(c, g, ws.tskinny, st))) return rc;
    if ((rc = run_rmsnorm<T>(c, ws.tNrm, ws.tX, lw.ffn_norm, Mt, 0, st))) return rc;
    g = GemmArgs{};
    g.A = ws.tNrm; g.W[0] = lw.w_gate; g.W[1] = lw.w_up; g.n_seg = 2; g.segN = F; g.C = ws.tACT; g.M = Mt; g.K = H;
    g.epilogue = EPI_SWIGLU; g.a_rows = ws.t_a_rows;
    if ((rc = run_gemm<T>(c, g, ws.tskinny, st))) return rc;
    g = GemmArgs{};
    g.A = ws.tACT; g.W[0] = lw.w_down; g.n_seg = 1; g.segN = H; g.C = ws.tX; g.M = Mt; g.K = F; g.epilogue = EPI_RESIDUAL; g.a_rows = ws.t_a_rows;
    return run_gemm<T>(c, g, ws.tskinny, st);
}

// `tail` (may be NULL): the rows whose final hidden state the caller reads.  Where use_tail() holds, the last layer
// is run in its tail form and the result of those rows is in ws.tX (packed), not in ws.X.
template <typename T>
static int run_layers(const vla_model *m, const Workspace &ws, const RowsArgs &ra, const KvView &kv,
                      bool kv_single_layer, hipStream_t st, const TailSpec *tail = nullptr, float *keep = nullptr) {
    const vla_config &c = m->cfg;
    int H = c.hidden, F = c.ffn, M = ra.n_seq * ra.R, d = H / c.n_heads, rc;
    if ((rc = launch_rope_table(ws.rope, ra.R, ra.pos0, d, c.rope_theta, st))) return rc;
    // k-blocked operands: repacked weights present, a multi-row forward, every fast path available and the
    // 32-bit offsets of the loads sufficient
    const bool kb = !m->packed.empty() && ra.R > 1 && kblocked_shape_ok(c) && force_generic() == 0 &&
                    ws.vt && (size_t)ra.n_seq * c.n_heads <= 65535 && M >= 1 &&
                    (size_t)ws.a_rows * (F > H ? F : H) * 2 < ((size_t)1 << 31);
    // Single-row bf16 forwards: the split-K GEMMs leave their partial sums to the kernel that follows (rotation + KV
    // write after the QKV projection, residual add + next RMSNorm after the O and down projections), which adds them
    // in the order the stand-alone reduction would.
    const bool fuse_reduce = c.dtype == VLA_DTYPE_BF16 && ra.R == 1 && ws.skinny && !(force_generic() & (2 | 16)) &&
                             H % 1024 == 0 && H <= 8192;
    bool have_nrm = false;                 // the previous layer's down projection already wrote this layer's Nrm
    const bool tail_form = use_tail(tail, ra.R) && ws.tail_rows == tail->count && ra.R > 1;
    for (int l = 0; l < c.n_layers; l++) {
        const vla_layer_weights &lw = m->layers[l];
        int kl = kv_single_layer ? 0 : l;
        // keep: the caller wants the residual stream at the input of every layer
        if (keep && hipMemcpyAsync(keep + (size_t)l * M * H, ws.X, (size_t)M * H * 4, hipMemcpyDeviceToDevice, st) != hipSuccess) {
            vla_set_error("copy of the residual stream failed");
            return VLA_EHIP;
        }
        if (tail_form && l == c.n_layers - 1) return run_last_layer_tail<T>(m, ws, ra, kv, l, kl, *tail, kb, st);
        if (kb) {
            if ((rc = run_layer_kblocked(m, ws, ra, kv, l, kl, st))) return rc;
            continue;
        }
        if (!have_nrm && (rc = run_rmsnorm<T>(c, ws.Nrm, ws.X, lw.attn_norm, M, 0, st))) return rc;
        have_nrm = false;
        // single-row forwards stream the weights from HBM: hand the GEMMs the repacked copies as well, where they exist
        const vla_layer_weights *pk = (ra.R == 1 && !m->packed.empty() && kblocked_shape_ok(c)) ? &m->packed[l] : nullptr;
        int ds = 0;
        GemmArgs g{};
        g.A = ws.Nrm; g.W[0] = lw.wq; g.W[1] = lw.wk; g.W[2] = lw.wv; g.n_seg = 3; g.segN = H;
        g.C = ws.QKV; g.M = M; g.K = H; g.epilogue = EPI_STORE; g.a_rows = ws.a_rows;
        if (pk) { g.Wkb[0] = pk->wq; g.Wkb[1] = pk->wk; g.Wkb[2] = pk->wv; }
        // multi-row bf16 forwards at head_dim 128: rotation and KV write ride the projection's epilogue
        int fused = 0;
        if (c.dtype == VLA_DTYPE_BF16 && ra.R > 1 && d == 128 && !(force_generic() & (1 | 16))) {
            QkvRopeArgs qa{ws.Q, ws.rope, &kv, kl, &ra};
            GemmArgs gf = g;
            gf.epilogue = EPI_QKV_ROPE; gf.rope = &qa;
            fused = try_gemm_bf16_large(gf, st);
            if (fused < 0) return fused;
        }
        if (!fused) {
            if (fuse_reduce) g.deferred_splits = &ds;
            if ((rc = run_gemm<T>(c, g, ws.skinny, st))) return rc;
            if (c.dtype == VLA_DTYPE_BF16 && !(force_generic() & 16))
                rc = launch_rope_kv_write_bf16((bf16_t *)ws.Q, ds ? (const float *)ws.skinny : ws.QKV, ds ? ds : 1, (size_t)M * 3 * H,
                                               ws.rope, kv, kl, ra, H, st);
            else rc = launch_rope_kv_write<T>((T *)ws.Q, ws.QKV, ws.rope, kv, kl, ra, H, st);
            if (rc) return rc;
        }
        int done = 0;
        if (c.dtype == VLA_DTYPE_BF16) {
            if (ra.R == 1)
                done = (force_generic() & 8) ? 0 : try_attention_decode_bf16((bf16_t *)ws.AO, (const bf16_t *)ws.Q, kv, kl, ra, H, st);
            else
                done = (force_generic() & 4) ? 0 : try_attention_prefill_bf16((bf16_t *)ws.AO, (const bf16_t *)ws.Q, kv, kl, ra, H, ws.vt, 0, st);
            if (done < 0) return done;
        }
        if (!done && (rc = launch_attention_generic<T>((T *)ws.AO, (const T *)ws.Q, kv, kl, ra, H, st))) return rc;
        g = GemmArgs{};
        g.A = ws.AO; g.W[0] = lw.wo; g.n_seg = 1; g.segN = H; g.C = ws.X; g.M = M; g.K = H; g.epilogue = EPI_RESIDUAL; g.a_rows = ws.a_rows;
        ds = 0;
        if (fuse_reduce) g.deferred_splits = &ds;
        if ((rc = run_gemm<T>(c, g, ws.skinny, st))) return rc;
        if (ds) {
            rc = try_reduce_residual_rmsnorm_bf16((bf16_t *)ws.Nrm, ws.X, (const float *)ws.skinny, ds, M, H, (const float *)lw.ffn_norm, c.rms_eps, st);
            if (rc == 0) { vla_set_error("internal: fused reduction declined"); return VLA_ESHAPE; }
            if (rc < 0) return rc;
        } else if ((rc = run_rmsnorm<T>(c, ws.Nrm, ws.X, lw.ffn_norm, M, 0, st))) return rc;
        g = GemmArgs{};
        g.A = ws.Nrm; g.W[0] = lw.w_gate; g.W[1] = lw.w_up; g.n_seg = 2; g.segN = F; g.C = ws.ACT; g.M = M; g.K = H;
        g.epilogue = EPI_SWIGLU; g.a_rows = ws.a_rows;
        if (pk) { g.Wkb[0] = pk->w_gate; g.Wkb[1] = pk->w_up; }
        if ((rc = run_gemm<T>(c, g, ws.skinny, st))) return rc;
        g = GemmArgs{};
        g.A = ws.ACT; g.W[0] = lw.w_down; g.n_seg = 1; g.segN = H; g.C = ws.X; g.M = M; g.K = F; g.epilogue = EPI_RESIDUAL; g.a_rows = ws.a_rows;
        ds = 0;
        if (fuse_reduce) g.deferred_splits = &ds;
        if ((rc = run_gemm<T>(c, g, ws.skinny, st))) return rc;
        if (ds) {
            const float *next_gain = l + 1 < c.n_layers ? (const float *)m->layers[l + 1].attn_norm : nullptr;
            rc = try_reduce_residual_rmsnorm_bf16((bf16_t *)ws.Nrm, ws.X, (const float *)ws.skinny, ds, M, H, next_gain, c.rms_eps, st);
            if (rc == 0) { vla_set_error("internal: fused reduction declined"); return VLA_ESHAPE; }
            if (rc < 0) return rc;
            have_nrm = next_gain != nullptr;
        }
    }
    return 0;
}

int vla_check_config(const vla_config *c) { return check_config(c); }
int vla_check_rows_per_pass(const vla_config &c, long n_seq, long rows_per_seq) { return check_rows_per_pass(c, n_seq, rows_per_seq); }
int vla_gemm_dispatch(const vla_config &c, const GemmArgs &g, hipStream_t st) {
    return c.dtype == VLA_DTYPE_F32 ? run_gemm<float>(c, g, nullptr, st) : run_gemm<bf16_t>(c, g, nullptr, st);
}

static int prefill_tail_rows(int S) { const TailSpec t{S - 1, 1}; return use_tail(&t, S) ? 1 : 0; }
// recompute, autoregressive mode: rows S - 1 .. S + A - 2 are read (the value head reads the first of them)
static int recompute_tail_rows(int S, int A, int mode) {
    const TailSpec t{S - 1, A};
    return mode == VLA_MODE_AR && use_tail(&t, S + A - 1) ? A : 0;
}

static KvView kv_view(const vla_config &c, void *kv, int n_seq, int n_layers) {
    KvView v;
    v.layer_elems = kv_layer_elems(c, n_seq);
    v.k = kv;
    v.v = (char *)kv + (size_t)n_layers * v.layer_elems * elt_size(c);
    v.n_seq = n_seq; v.n_heads = c.n_heads; v.d = c.hidden / c.n_heads; v.pos_stride = c.max_seq;
    return v;
}

// ------------------------------------------------------------------------------------------ entry bodies
template <typename T>
static int prefill_impl(vla_model *m, void *kvbuf, void *wsbuf, const void *patch, const int32_t *ids, int B,
                        int P, int T_, float *h_last, float *value, hipStream_t st) {
    const vla_config &c = m->cfg;
    int S = P + T_, H = c.hidden, rc;
    const TailSpec tail{S - 1, 1};                    // only the last prefix row is read after the last layer
    const bool tf = use_tail(&tail, S);
    Workspace ws = plan_workspace(c, (char *)wsbuf, B, S, S, 0, false, tf ? 1 : 0);
    if ((rc = launch_embed_prefix<T>(ws.X, (const T *)patch, ids, (const T *)m->w.embed, B, P, T_, S, H, c.vocab, st))) return rc;
    RowsArgs ra{B, S, 0, 0x7fffffff};
    KvView kv = kv_view(c, kvbuf, B, c.n_layers);
    if ((rc = run_layers<T>(m, ws, ra, kv, false, st, &tail))) return rc;
    if (tf) rc = launch_final_norm_rows(h_last, ws.tX, (const float *)m->w.final_norm, B, 1, 0, 1, H, c.rms_eps, st);
    else rc = launch_final_norm_rows(h_last, ws.X, (const float *)m->w.final_norm, B, S, S - 1, 1, H, c.rms_eps, st);
    if (rc) return rc;
    if (value && (rc = launch_value_head(value, h_last, (const float *)m->w.value_w, m->w.value_b, (const float *)m->w.value_bias, value_dim(m->cfg), B, H, H, st))) return rc;
    return 0;
}

template <typename T>
static int decode_impl(vla_model *m, void *kvbuf, void *wsbuf, const float *h_last, int B, int S, int A, int mode,
                       const void *slot_embed, float temperature, const float *gumbel, int32_t *bins, float *logp,
                       float *entropy, float *logits, hipStream_t st) {
    const vla_config &c = m->cfg;
    int H = c.hidden, rc;
    const T *head = (const T *)m->w.lm_head + (size_t)(c.vocab - VLA_N_BINS) * H;
    KvView kv = kv_view(c, kvbuf, B, c.n_layers);
    if (mode == VLA_MODE_AR) {
        Workspace ws = plan_workspace(c, (char *)wsbuf, B, 1, S + A, B, false);
        const float *h = h_last;
        for (int j = 0; j < A; j++) {
            bool more = j + 1 < A;
            if ((rc = launch_head_sample<T>(h, head, B, H, temperature, gumbel, nullptr, bins, logp, entropy, logits, A, j,
                                            more ? ws.X : nullptr, (const T *)m->w.embed, c.vocab, st))) return rc;
            if (!more) break;
            RowsArgs ra{B, 1, S + j, 0x7fffffff};
            if ((rc = run_layers<T>(m, ws, ra, kv, false, st))) return rc;
            if ((rc = launch_final_norm_rows(ws.Hb, ws.X, (const float *)m->w.final_norm, B, 1, 0, 1, H, c.rms_eps, st))) return rc;
            h = ws.Hb;
        }
    } else {
        Workspace ws = plan_workspace(c, (char *)wsbuf, B, A, S + A, B * A, false);
        if ((rc = launch_embed_slots<T>(ws.X, (const T *)slot_embed, B, A, A, 0, H, st))) return rc;
        RowsArgs ra{B, A, S, S};
        if ((rc = run_layers<T>(m, ws, ra, kv, false, st))) return rc;
        if ((rc = launch_final_norm_rows(ws.Hb, ws.X, (const float *)m->w.final_norm, B, A, 0, A, H, c.rms_eps, st))) return rc;
        if ((rc = launch_head_sample<T>(ws.Hb, head, B * A, H, temperature, gumbel, nullptr, bins, logp, entropy, logits, 1, 0,
                                        nullptr, (const T *)nullptr, c.vocab, st))) return rc;
    }
    return 0;
}

template <typename T>
static int recompute_impl(vla_model *m, void *wsbuf, const void *patch, const int32_t *ids, const int32_t *bins, int N,
                          int P, int T_, int A, int mode, const void *slot_embed, float temperature, float *logp,
                          float *entropy, float *value, float *logits, hipStream_t st) {
    const vla_config &c = m->cfg;
    int S = P + T_, H = c.hidden, rc;
    int R = (mode == VLA_MODE_AR) ? S + A - 1 : S + A;
    int first = (mode == VLA_MODE_AR) ? S - 1 : S;          // row that predicts action token 1
    int mb = recompute_micro_batch(c, N, S + A);
    const T *head = (const T *)m->w.lm_head + (size_t)(c.vocab - VLA_N_BINS) * H;
    const int tr = recompute_tail_rows(S, A, mode);
    const TailSpec tail{S - 1, A};
    Workspace ws = plan_workspace(c, (char *)wsbuf, mb, R, R, mb * (A + 1), true, tr);
    for (int n0 = 0; n0 < N; n0 += mb) {
        int n = (N - n0 < mb) ? N - n0 : mb;
        const T *pp = (const T *)patch + (size_t)n0 * P * H;
        if ((rc = launch_embed_prefix<T>(ws.X, pp, ids + (size_t)n0 * T_, (const T *)m->w.embed, n, P, T_, R, H, c.vocab, st))) return rc;
        if (mode == VLA_MODE_AR) {
            if ((rc = launch_embed_tokens<T>(ws.X, bins + (size_t)n0 * A, A, A - 1, (const T *)m->w.embed, n, R, S, H, c.vocab, st))) return rc;
        } else {
            if ((rc = launch_embed_slots<T>(ws.X, (const T *)slot_embed, n, A, R, S, H, st))) return rc;
        }
        RowsArgs ra{n, R, 0, (mode == VLA_MODE_AR) ? 0x7fffffff : S};
        KvView kv;
        kv.layer_elems = kv_layer_elems(c, mb);
        kv.k = ws.kvs_k; kv.v = ws.kvs_v; kv.n_seq = n; kv.n_heads = c.n_heads; kv.d = H / c.n_heads; kv.pos_stride = c.max_seq;
        if ((rc = run_layers<T>(m, ws, ra, kv, true, st, tr ? &tail : nullptr))) return rc;
        // after a tail-form last layer the read-out rows are the packed tail rows 0 .. A - 1 of each rollout
        const float *Xh = tr ? ws.tX : ws.X;
        const int rows_h = tr ? A : R, first_h = tr ? 0 : first, value_row = tr ? 0 : S - 1;
        if ((rc = launch_final_norm_rows(ws.Hb, Xh, (const float *)m->w.final_norm, n, rows_h, first_h, A, H, c.rms_eps, st))) return rc;
        size_t o = (size_t)n0 * A;
        if ((rc = launch_head_sample<T>(ws.Hb, head, n * A, H, temperature, nullptr, bins + o, nullptr, logp + o, entropy + o,
                                        logits ? logits + o * VLA_N_BINS : nullptr, 1, 0, nullptr, (const T *)nullptr, c.vocab, st))) return rc;
        if (value) {
            float *hv = ws.Hb + (size_t)mb * A * H;
            if ((rc = launch_final_norm_rows(hv, Xh, (const float *)m->w.final_norm, n, rows_h, value_row, 1, H, c.rms_eps, st))) return rc;
            if ((rc = launch_value_head(value + (size_t)n0 * value_dim(m->cfg), hv, (const float *)m->w.value_w, m->w.value_b, (const float *)m->w.value_bias, value_dim(m->cfg), n, H, H, st))) return rc;
        }
    }
    return 0;
}

size_t vla_forward_streams_bytes(const vla_config &c, int n_max, int R) {
    return plan_workspace(c, nullptr, n_max, R, R, 0, true, 0).total;
}

template <typename T>
static int forward_streams_impl(vla_model *m, void *fw_ws, int n_max, const void *patch, const int32_t *ids, const int32_t *bins, int n,
                                int P, int T_, int A, int mode, const void *slot_embed, float *keep, const float **x_final, hipStream_t st) {
    const vla_config &c = m->cfg;
    const int S = P + T_, H = c.hidden, R = (mode == VLA_MODE_AR) ? S + A - 1 : S + A;
    int rc;
    Workspace ws = plan_workspace(c, (char *)fw_ws, n_max, R, R, 0, true, 0);
    if ((rc = launch_embed_prefix<T>(ws.X, (const T *)patch, ids, (const T *)m->w.embed, n, P, T_, R, H, c.vocab, st))) return rc;
    if (mode == VLA_MODE_AR) {
        if ((rc = launch_embed_tokens<T>(ws.X, bins, A, A - 1, (const T *)m->w.embed, n, R, S, H, c.vocab, st))) return rc;
    } else if ((rc = launch_embed_slots<T>(ws.X, (const T *)slot_embed, n, A, R, S, H, st))) return rc;
    RowsArgs ra{n, R, 0, (mode == VLA_MODE_AR) ? 0x7fffffff : S};
    KvView kv;
    kv.layer_elems = kv_layer_elems(c, n_max);
    kv.k = ws.kvs_k; kv.v = ws.kvs_v; kv.n_seq = n; kv.n_heads = c.n_heads; kv.d = H / c.n_heads; kv.pos_stride = c.max_seq;
    if ((rc = run_layers<T>(m, ws, ra, kv, true, st, nullptr, keep))) return rc;
    *x_final = ws.X;
    return 0;
}

int vla_forward_streams(vla_model *m, void *fw_ws, int n_max, const void *patch, const int32_t *ids, const int32_t *bins, int n,
                        int P, int T, int A, int mode, const void *slot_embed, float *keep, const float **x_final, hipStream_t st) {
    return m->cfg.dtype == VLA_DTYPE_F32
               ? forward_streams_impl<float>(m, fw_ws, n_max, patch, ids, bins, n, P, T, A, mode, slot_embed, keep, x_final, st)
               : forward_streams_impl<bf16_t>(m, fw_ws, n_max, patch, ids, bins, n, P, T, A, mode, slot_embed, keep, x_final, st);
}

// ------------------------------------------------------------------------------------------ C ABI
extern "C" {

int vla_version(void) { return VLA_VERSION; }

const char *vla_last_error(void) { return g_err; }

int vla_create(const vla_config *cfg, const vla_weights *w, vla_model **out) {
    if (!out) { vla_set_error("out is NULL"); return VLA_EINVAL; }
    *out = nullptr;
    int rc = check_config(cfg);
    if (rc) return rc;
    if (!w || !w->embed || !w->lm_head || !w->final_norm || !w->layers) {
        vla_set_error("weights, embed, lm_head, final_norm or layers is NULL");
        return VLA_EINVAL;
    }
    for (int l = 0; l < cfg->n_layers; l++) {
        const vla_layer_weights &lw = w->layers[l];
        if (!lw.attn_norm || !lw.wq || !lw.wk || !lw.wv || !lw.wo || !lw.ffn_norm || !lw.w_gate || !lw.w_up || !lw.w_down) {
            vla_set_error("layer %d has a NULL weight pointer", l);
            return VLA_EINVAL;
        }
    }
    vla_model *m = new (std::nothrow) vla_model;
    if (!m) { vla_set_error("out of host memory"); return VLA_EINVAL; }
    m->cfg = *cfg;
    m->w = *w;
    m->layers.assign(w->layers, w->layers + cfg->n_layers);
    m->w.layers = m->layers.data();
    *out = m;
    return VLA_OK;
}

size_t vla_prepack_bytes(const vla_config *cfg) {
    if (check_config(cfg) != VLA_OK) return 0;
    if (!kblocked_shape_ok(*cfg)) return 0;
    return prepack_layer_bytes(*cfg) * cfg->n_layers;
}

int vla_prepack(vla_model *m, void *buffer, size_t bytes, void *stream) {
    if (!m) { vla_set_error("model is NULL"); return VLA_EINVAL; }
    if (!buffer) { m->packed.clear(); return VLA_OK; }
    const vla_config &c = m->cfg;
    if (!kblocked_shape_ok(c)) { m->packed.clear(); return VLA_OK; }       // nothing to repack for this shape
    const size_t need = prepack_layer_bytes(c) * c.n_layers;
    if (bytes < need) { vla_set_error("prepack buffer of %zu bytes, %zu needed", bytes, need); return VLA_EWORKSPACE; }
    if ((uintptr_t)buffer % 256 != 0) { vla_set_error("prepack buffer must be 256-byte aligned"); return VLA_EINVAL; }
    hipStream_t st = (hipStream_t)stream;
    std::vector<vla_layer_weights> packed(c.n_layers);
    bf16_t *dst = (bf16_t *)buffer;
    const int H = c.hidden, F = c.ffn;
    int rc;
    for (int l = 0; l < c.n_layers; l++) {
        const vla_layer_weights &lw = m->layers[l];
        vla_layer_weights pk = lw;                                         // norm gains stay as they are
        struct { const void *src; const void **slot; int N, K; } mats[7] = {
            {lw.wq, &pk.wq, H, H}, {lw.wk, &pk.wk, H, H}, {lw.wv, &pk.wv, H, H}, {lw.wo, &pk.wo, H, H},
            {lw.w_gate, &pk.w_gate, F, H}, {lw.w_up, &pk.w_up, F, H}, {lw.w_down, &pk.w_down, H, F}};
        for (auto &mt : mats) {
            if ((rc = launch_weight_kblock(dst, (const bf16_t *)mt.src, mt.N, mt.K, st))) return rc;
            *mt.slot = dst;
            dst += (size_t)(mt.N + VLA_KB_PAD_ROWS) * mt.K;
        }
        packed[l] = pk;
    }
    m->packed.swap(packed);
    return VLA_OK;
}

int vla_destroy(vla_model *m) {
    if (!m) { vla_set_error("model is NULL"); return VLA_EINVAL; }
    delete m;
    return VLA_OK;
}

size_t vla_kv_bytes(const vla_config *cfg, int B, int max_pos) {
    if (check_config(cfg)) return 0;
    if (B <= 0 || max_pos <= 0) { vla_set_error("B and max_pos must be positive"); return 0; }
    if (B > cfg->max_batch || max_pos > cfg->max_seq) {
        vla_set_error("B %d / max_pos %d exceed capacity %d / %d", B, max_pos, cfg->max_batch, cfg->max_seq);
        return 0;
    }
    return 2 * (size_t)cfg->n_layers * kv_layer_elems(*cfg, B) * elt_size(*cfg);
}

size_t vla_workspace_bytes(const vla_config *cfg, int entry, int B, int S, int A) {
    if (check_config(cfg)) return 0;
    if (B <= 0 || S <= 0 || A < 0) { vla_set_error("B, S must be positive and A non-negative"); return 0; }
    int a = A > 0 ? A : 1;
    switch (entry) {
        case VLA_ENTRY_PREFILL:
            if (B > cfg->max_batch || S > cfg->max_seq) { vla_set_error("B or S exceeds capacity"); return 0; }
            if (check_rows_per_pass(*cfg, B, S)) return 0;
            return plan_workspace(*cfg, nullptr, B, S, S, 0, false, prefill_tail_rows(S)).total;
        case VLA_ENTRY_DECODE: {
            if (B > cfg->max_batch || S + a > cfg->max_seq + 1) { vla_set_error("B or S + A exceeds capacity"); return 0; }
            if (check_rows_per_pass(*cfg, B, a)) return 0;
            size_t ar = plan_workspace(*cfg, nullptr, B, 1, S + a, B, false).total;
            size_t ch = (S + a <= cfg->max_seq) ? plan_workspace(*cfg, nullptr, B, a, S + a, B * a, false).total : 0;
            return ar > ch ? ar : ch;
        }
        case VLA_ENTRY_RECOMPUTE: {
            if (S + a > cfg->max_seq + 1) { vla_set_error("S + A exceeds capacity"); return 0; }
            int R = (S + a <= cfg->max_seq) ? S + a : S + a - 1;
            int mb = recompute_micro_batch(*cfg, B, S + a);
            // (the query does not know the mode: the autoregressive form's tail buffers are included either way)
            return plan_workspace(*cfg, nullptr, mb, R, R, mb * (a + 1), true, recompute_tail_rows(S, a, VLA_MODE_AR)).total;
        }
        default:
            vla_set_error("unknown entry %d", entry);
            return 0;
    }
}

int vla_prefill(vla_model *m, void *kv, void *ws, size_t ws_bytes, const void *patch, const int32_t *ids, int B, int P,
                int T, float *h_last, float *value, void *stream) {
    if (!m || !kv || !ws || !h_last) { vla_set_error("model, kv, ws or h_last is NULL"); return VLA_EINVAL; }
    if (B <= 0 || P < 0 || T < 0 || P + T < 1) { vla_set_error("need B >= 1, P, T >= 0, P + T >= 1"); return VLA_EINVAL; }
    if ((P > 0 && !patch) || (T > 0 && !ids)) { vla_set_error("patch / ids is NULL"); return VLA_EINVAL; }
    if (value && !m->w.value_w) { vla_set_error("value requested but the model has no value head"); return VLA_EINVAL; }
    const vla_config &c = m->cfg;
    if (B > c.max_batch || P + T > c.max_seq) {
        vla_set_error("B %d / S %d exceed capacity %d / %d", B, P + T, c.max_batch, c.max_seq);
        return VLA_ESHAPE;
    }
    if (int rc = check_rows_per_pass(c, B, P + T)) return rc;
    size_t need = plan_workspace(c, nullptr, B, P + T, P + T, 0, false, prefill_tail_rows(P + T)).total;
    if (ws_bytes < need) { vla_set_error("workspace %zu bytes, need %zu", ws_bytes, need); return VLA_EWORKSPACE; }
    hipStream_t st = (hipStream_t)stream;
    return c.dtype == VLA_DTYPE_F32 ? prefill_impl<float>(m, kv, ws, patch, ids, B, P, T, h_last, value, st)
                                    : prefill_impl<bf16_t>(m, kv, ws, patch, ids, B, P, T, h_last, value, st);
}

int vla_decode_actions(vla_model *m, void *kv, void *ws, size_t ws_bytes, const float *h_last, int B, int S, int A,
                       int mode, const void *slot_embed, float temperature, const float *gumbel, int32_t *bins,
                       float *logp, float *entropy, float *logits, void *stream) {
    if (!m || !kv || !ws || !bins || !logp || !entropy) { vla_set_error("model, kv, ws, bins, logp or entropy is NULL"); return VLA_EINVAL; }
    if (mode != VLA_MODE_AR && mode != VLA_MODE_PARALLEL_CHUNK) { vla_set_error("unknown mode %d", mode); return VLA_EINVAL; }
    if (B <= 0 || S <= 0 || A <= 0) { vla_set_error("B, S, A must be positive"); return VLA_EINVAL; }
    if (!(temperature > 0.f)) { vla_set_error("temperature must be positive"); return VLA_EINVAL; }
    if (mode == VLA_MODE_AR && !h_last) { vla_set_error("h_last is NULL"); return VLA_EINVAL; }
    if (mode == VLA_MODE_PARALLEL_CHUNK && !slot_embed) { vla_set_error("slot_embed is NULL"); return VLA_EINVAL; }
    const vla_config &c = m->cfg;
    int rows = (mode == VLA_MODE_AR) ? S + A - 1 : S + A;
    if (B > c.max_batch || rows > c.max_seq) {
        vla_set_error("B %d / positions %d exceed capacity %d / %d", B, rows, c.max_batch, c.max_seq);
        return VLA_ESHAPE;
    }
    if (int rc = check_rows_per_pass(c, B, mode == VLA_MODE_AR ? 1 : A)) return rc;
    size_t need = (mode == VLA_MODE_AR) ? plan_workspace(c, nullptr, B, 1, S + A, B, false).total
                                        : plan_workspace(c, nullptr, B, A, S + A, B * A, false).total;
    if (ws_bytes < need) { vla_set_error("workspace %zu bytes, need %zu", ws_bytes, need); return VLA_EWORKSPACE; }
    hipStream_t st = (hipStream_t)stream;
    return c.dtype == VLA_DTYPE_F32
               ? decode_impl<float>(m, kv, ws, h_last, B, S, A, mode, slot_embed, temperature, gumbel, bins, logp, entropy, logits, st)
               : decode_impl<bf16_t>(m, kv, ws, h_last, B, S, A, mode, slot_embed, temperature, gumbel, bins, logp, entropy, logits, st);
}

int vla_logprob_recompute(vla_model *m, void *ws, size_t ws_bytes, const void *patch, const int32_t *ids,
                          const int32_t *bins, int N, int P, int T, int A, int mode, const void *slot_embed,
                          float temperature, float *logp, float *entropy, float *value, float *logits, void *stream) {
    if (!m || !ws || !bins || !logp || !entropy) { vla_set_error("model, ws, bins, logp or entropy is NULL"); return VLA_EINVAL; }
    if (mode != VLA_MODE_AR && mode != VLA_MODE_PARALLEL_CHUNK) { vla_set_error("unknown mode %d", mode); return VLA_EINVAL; }
    if (N <= 0 || P < 0 || T < 0 || P + T < 1 || A <= 0) { vla_set_error("need N, A >= 1, P, T >= 0, P + T >= 1"); return VLA_EINVAL; }
    if ((P > 0 && !patch) || (T > 0 && !ids)) { vla_set_error("patch / ids is NULL"); return VLA_EINVAL; }
    if (!(temperature > 0.f)) { vla_set_error("temperature must be positive"); return VLA_EINVAL; }
    if (mode == VLA_MODE_PARALLEL_CHUNK && !slot_embed) { vla_set_error("slot_embed is NULL"); return VLA_EINVAL; }
    if (value && !m->w.value_w) { vla_set_error("value requested but the model has no value head"); return VLA_EINVAL; }
    const vla_config &c = m->cfg;
    int S = P + T, R = (mode == VLA_MODE_AR) ? S + A - 1 : S + A;
    if (R > c.max_seq) { vla_set_error("rows per rollout %d exceed max_seq %d", R, c.max_seq); return VLA_ESHAPE; }
    int mb = recompute_micro_batch(c, N, S + A);
    size_t need = plan_workspace(c, nullptr, mb, R, R, mb * (A + 1), true, recompute_tail_rows(S, A, mode)).total;
    if (ws_bytes < need) { vla_set_error("workspace %zu bytes, need %zu", ws_bytes, need); return VLA_EWORKSPACE; }
    hipStream_t st = (hipStream_t)stream;
    return c.dtype == VLA_DTYPE_F32
               ? recompute_impl<float>(m, ws, patch, ids, bins, N, P, T, A, mode, slot_embed, temperature, logp, entropy, value, logits, st)
               : recompute_impl<bf16_t>(m, ws, patch, ids, bins, N, P, T, A, mode, slot_embed, temperature, logp, entropy, value, logits, st);
}

int vla_debug_force_generic(int mask) {
    if (mask < 0 || mask > 31) { vla_set_error("force_generic mask %d outside 0..31", mask); return VLA_EINVAL; }
    g_force_generic = mask;
    return VLA_OK;
}

int vla_profile_enable(int on) {
    prof_clear();
    g_prof_on = on != 0;
    return VLA_OK;
}

int vla_profile_report(char *buf, size_t n) {
    if (!buf || n == 0) { vla_set_error("buf is NULL or empty"); return VLA_EINVAL; }
    struct Agg { const char *label; long count; double ms, work; };
    std::vector<Agg> agg;
    for (auto &r : g_prof) {
        if (hipEventSynchronize(r.e1) != hipSuccess) { vla_set_error("hipEventSynchronize failed"); return VLA_EHIP; }
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.e0, r.e1) != hipSuccess) { vla_set_error("hipEventElapsedTime failed"); return VLA_EHIP; }
        Agg *a = nullptr;
        for (auto &x : agg) if (strcmp(x.label, r.label) == 0) { a = &x; break; }
        if (!a) { agg.push_back(Agg{r.label, 0, 0.0, 0.0}); a = &agg.back(); }
        a->count++; a->ms += ms; a->work += r.work;
    }
    size_t off = 0;
    buf[0] = 0;
    for (auto &a : agg) {
        int w = snprintf(buf + off, n - off, "%s %ld %.6f %.6e\n", a.label, a.count, a.ms, a.work);
        if (w < 0 || (size_t)w >= n - off) break;
        off += (size_t)w;
    }
    return (int)agg.size();
}

}  // extern "C"
