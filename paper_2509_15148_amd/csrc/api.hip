// C ABI: error reporting, the target-model handle, workspace carving and the launch sequence of
// atts_score_drafts, plus the stand-alone stage entry points.  Host code only; kernels live in
// gemm.hip / attention.hip / elementwise.hip / calib.hip.
#include "common.h"

#include <algorithm>

#include <stdarg.h>
#include <stdio.h>
#include <mutex>
#include <new>
#include <vector>

struct atts_model {
    atts_model_desc desc;
    const void* tok_embed;
    const float* final_norm;
    const void* lm_head;
    std::vector<const float*> attn_norm, ffn_norm;
    std::vector<const void*> wqkv, wo, w_gate_up, w_down;
    int32_t* err_flag;   // device
};

// Keys and values of a prompt prefix, kept per layer as the attention kernels read them (keys after RoPE as rows,
// values transposed for the MFMA attention kernel, else as rows), plus the hidden state of its last row.
struct atts_prefix {
    const atts_model* model;
    int32_t capacity;     // rows the caches can hold
    int32_t P;            // rows held
    int64_t cap_ld;       // row pitch of the transposed-value cache (capacity rounded up to 64)
    bool uses_vt;
    char* k_cache;        // [L][capacity][n_kv hd]
    char* v_cache;        // uses_vt: [L][n_kv hd][cap_ld]   else: [L][capacity][n_kv hd]
    float* h_last;        // [d_model]
};

namespace atts {

static thread_local char g_error[512] = "";

int32_t fail(int32_t code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
    return code;
}

// ---- stage timing ---------------------------------------------------------------------------
namespace {
struct ProfRecord {
    int32_t stage;
    hipEvent_t start, stop;
};
bool g_prof_on = false;
std::vector<ProfRecord> g_prof;
}  // namespace

StageTimer::StageTimer(int32_t stage, hipStream_t s) : st_(s), stage_(stage) {
    if (!g_prof_on) return;
    if (hipEventCreate(&start_) != hipSuccess) return;
    if (hipEventCreate(&stop_) != hipSuccess) {
        (void)hipEventDestroy(start_);
        return;
    }
    (void)hipEventRecord(start_, st_);
    live_ = true;
}
StageTimer::~StageTimer() {
    if (!live_) return;
    (void)hipEventRecord(stop_, st_);
    g_prof.push_back(ProfRecord{stage_, start_, stop_});
}

namespace {

void prof_clear() {
    for (auto& r : g_prof) {
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    g_prof.clear();
}

// Sub-buffers of the scoring workspace, each 256-byte aligned.
struct Workspace {
    size_t h, xn, qkv, kpart, vt, ao, act, rope, xs, targets, valid, partials, zt, lp, total;
    int64_t ldv;
    int32_t n_part;
};

// GEMM inputs of the bf16 path are allocated in whole tiles (768 rows = a multiple of both tile heights): the
// aligned kernel then serves every row count (it reads the pad rows, whatever they hold, and drops their results).
bool pads_rows(const atts_model_desc& d) { return d.dtype == ATTS_DTYPE_BF16; }
constexpr int kSplitQkvRows = 128;

// K-split projections (few rows, narrow output) store one partial result per K slice; the three of a layer (QKV, O,
// down) use the same buffer one after the other.  Slices per projection for M rows through the model:
struct SplitPlan {
    int32_t qkv, o, down;        // 1 = not split (direct epilogue)
    size_t bytes;                // of the shared partial buffer
};
SplitPlan split_plan(const atts_model_desc& d, int64_t M) {
    SplitPlan p{1, 1, 1, 0};
    if (M < 1 || M > (1 << 24)) return p;
    const int32_t qd = d.n_q_heads * d.head_dim, qkv_out = (d.n_q_heads + 2 * d.n_kv_heads) * d.head_dim;
    const bool padded = pads_rows(d);
    if (M <= kSplitQkvRows) p.qkv = gemm_partial_slices(d.dtype, (int32_t)M, qkv_out, d.d_model, padded);
    p.o = gemm_partial_slices(d.dtype, (int32_t)M, d.d_model, qd, padded);
    p.down = gemm_partial_slices(d.dtype, (int32_t)M, d.d_model, d.d_ffn, padded);
    auto need = [&](int32_t slices, int64_t n) { return slices > 1 ? (size_t)slices * (size_t)M * (size_t)n * sizeof(float) : (size_t)0; };
    p.bytes = std::max(need(p.qkv, qkv_out), std::max(need(p.o, d.d_model), need(p.down, d.d_model)));
    return p;
}

Workspace carve(const atts_model_desc& d, ScoreShape s) {
    const size_t es = dtype_size(d.dtype);
    const size_t R = (size_t)s.R(), B = (size_t)s.B();
    // + one more block: with a cached prefix the GEMMs start at row P, not at row 0
    const size_t Ra = pads_rows(d) ? align_up(R, 768) + 768 : R, Ba = pads_rows(d) ? align_up(B, 768) : B;
    Workspace w{};
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t at = off;
        off += align_up(bytes, 256);
        return at;
    };
    w.h = take(R * d.d_model * sizeof(float));
    w.xn = take(Ra * d.d_model * es);
    w.qkv = take(R * (size_t)(d.n_q_heads + 2 * d.n_kv_heads) * d.head_dim * es);
    // partial sums of the K-split projections: the call computes all R rows, or the K T draft rows after a cached prefix
    w.kpart = take(std::max(split_plan(d, (int64_t)R).bytes, split_plan(d, (int64_t)B).bytes));
    w.ldv = (int64_t)align_up(R, 64);
    w.vt = take(attention_uses_vt(d.dtype, d.head_dim) ? (size_t)d.n_kv_heads * d.head_dim * w.ldv * es : 0);
    w.ao = take(Ra * (size_t)d.n_q_heads * d.head_dim * es);
    w.act = take(Ra * (size_t)d.d_ffn * es);
    w.rope = take(R * (size_t)(d.head_dim / 2) * sizeof(float2));
    w.xs = take(Ba * d.d_model * es);
    w.targets = take(B * sizeof(int32_t));
    w.valid = take(B);
    w.n_part = lmhead_num_partials(d.dtype, s.B(), d.vocab, d.d_model, pads_rows(d));
    w.partials = take(B * (size_t)w.n_part * sizeof(float2));
    w.zt = take(B * sizeof(float));
    w.lp = take(B * sizeof(float));
    w.total = off;
    return w;
}

int32_t check_score_shape(const char* fn, int32_t P, int32_t K, int32_t T) {
    if (P < 1 || K < 1 || T < 1) return fail(ATTS_ERR_INVALID_ARG, "%s: P = %d, K = %d, T_max = %d must all be >= 1", fn, P, K, T);
    if ((int64_t)P + T > (1 << 20)) return fail(ATTS_ERR_INVALID_ARG, "%s: P + T_max = %lld exceeds 1048576", fn, (long long)P + T);
    if ((int64_t)P + (int64_t)K * T > (1 << 24)) return fail(ATTS_ERR_INVALID_ARG, "%s: P + K T_max exceeds 2^24 rows", fn);
    return ATTS_OK;
}

#define ATTS_TRY(expr)                    \
    do {                                  \
        int32_t rc__ = (expr);            \
        if (rc__ != ATTS_OK) return rc__; \
    } while (0)

}  // namespace
}  // namespace atts

using namespace atts;

extern "C" {

const char* atts_last_error_string(void) { return g_error; }

int32_t atts_model_create(const atts_model_desc* desc, const atts_weights* w, atts_model** out) {
    if (!out) return fail(ATTS_ERR_INVALID_ARG, "atts_model_create: out is NULL");
    *out = nullptr;
    if (!desc || !w) return fail(ATTS_ERR_INVALID_ARG, "atts_model_create: desc / weights is NULL");
    const atts_model_desc& d = *desc;
    if (d.dtype != ATTS_DTYPE_F32 && d.dtype != ATTS_DTYPE_BF16)
        return fail(ATTS_ERR_INVALID_ARG, "atts_model_create: unknown dtype %d", d.dtype);
    if (d.n_layers < 0 || d.d_model < 1 || d.n_q_heads < 1 || d.n_kv_heads < 1 || d.head_dim < 2 || d.d_ffn < 1 || d.vocab < 1)
        return fail(ATTS_ERR_INVALID_ARG, "atts_model_create: non-positive dimension");
    if (d.n_q_heads % d.n_kv_heads) return fail(ATTS_ERR_SHAPE, "atts_model_create: n_kv_heads must divide n_q_heads");
    if (d.head_dim % 2 || d.head_dim > 256) return fail(ATTS_ERR_SHAPE, "atts_model_create: head_dim must be even and <= 256");
    const size_t es = dtype_size(d.dtype);
    if ((d.d_model * es) % 16 || (d.d_ffn * es) % 16 || ((size_t)d.n_q_heads * d.head_dim * es) % 16 || (d.head_dim * es) % 16)
        return fail(ATTS_ERR_SHAPE, "atts_model_create: d_model, d_ffn and head_dim rows must be multiples of 16 bytes");
    if (!(d.rms_eps >= 0.f) || !(d.rope_theta > 0.f)) return fail(ATTS_ERR_INVALID_ARG, "atts_model_create: bad rms_eps / rope_theta");
    if (!w->tok_embed || !w->final_norm || !w->lm_head) return fail(ATTS_ERR_INVALID_ARG, "atts_model_create: NULL embedding / final norm / LM head");
    if (d.n_layers > 0 && (!w->attn_norm || !w->wqkv || !w->wo || !w->ffn_norm || !w->w_gate_up || !w->w_down))
        return fail(ATTS_ERR_INVALID_ARG, "atts_model_create: NULL per-layer pointer array");
    atts_model* m = new (std::nothrow) atts_model();
    if (!m) return fail(ATTS_ERR_HIP, "atts_model_create: out of host memory");
    m->desc = d;
    m->tok_embed = w->tok_embed;
    m->final_norm = w->final_norm;
    m->lm_head = w->lm_head;
    for (int l = 0; l < d.n_layers; ++l) {
        if (!w->attn_norm[l] || !w->wqkv[l] || !w->wo[l] || !w->ffn_norm[l] || !w->w_gate_up[l] || !w->w_down[l]) {
            delete m;
            return fail(ATTS_ERR_INVALID_ARG, "atts_model_create: NULL weight pointer in layer %d", l);
        }
        if (((uintptr_t)w->wqkv[l] | (uintptr_t)w->wo[l] | (uintptr_t)w->w_gate_up[l] | (uintptr_t)w->w_down[l] |
             (uintptr_t)w->attn_norm[l] | (uintptr_t)w->ffn_norm[l]) & 15) {
            delete m;
            return fail(ATTS_ERR_INVALID_ARG, "atts_model_create: layer %d weights must be 16-byte aligned", l);
        }
        m->attn_norm.push_back(w->attn_norm[l]);
        m->wqkv.push_back(w->wqkv[l]);
        m->wo.push_back(w->wo[l]);
        m->ffn_norm.push_back(w->ffn_norm[l]);
        m->w_gate_up.push_back(w->w_gate_up[l]);
        m->w_down.push_back(w->w_down[l]);
    }
    if (((uintptr_t)w->tok_embed | (uintptr_t)w->lm_head | (uintptr_t)w->final_norm) & 15) {
        delete m;
        return fail(ATTS_ERR_INVALID_ARG, "atts_model_create: embedding / LM head / final norm must be 16-byte aligned");
    }
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&m->err_flag), sizeof(int32_t));
    if (e == hipSuccess) e = hipMemset(m->err_flag, 0, sizeof(int32_t));
    if (e != hipSuccess) {
        delete m;
        return fail(ATTS_ERR_HIP, "atts_model_create: device flag allocation failed: %s", hipGetErrorString(e));
    }
    *out = m;
    return ATTS_OK;
}

int32_t atts_model_destroy(atts_model* m) {
    if (!m) return ATTS_OK;
    (void)hipFree(m->err_flag);
    delete m;
    return ATTS_OK;
}

int32_t atts_workspace_bytes(const atts_model* m, int32_t P, int32_t K, int32_t T_max, size_t* out_bytes) {
    if (!m || !out_bytes) return fail(ATTS_ERR_INVALID_ARG, "atts_workspace_bytes: NULL argument");
    ATTS_TRY(check_score_shape("atts_workspace_bytes", P, K, T_max));
    *out_bytes = carve(m->desc, ScoreShape{P, K, T_max}).total;
    return ATTS_OK;
}

}  // extern "C"

namespace atts {
namespace {

// The forward pass over rows [row0, R) of the token tree s = [prefix (P) | K drafts of T].
//   row0 == 0:   everything is computed (pre == nullptr).
//   row0 == P:   keys / values of the prefix rows come from `pre` (pre->P == P), copied into the workspace before
//                each layer's attention.  save: the new rows' keys / values and the last row's hidden state are
//                appended to `pre` (K == 1: the new rows continue the prefix as one causal sequence).
// score: LM head + scores for the K T scoring rows (else the pass stops after the last layer).
// Where a continuation call keeps the keys / values of the whole token tree, per layer, as rows
// (rows [0, P) prefix, P + j Tc + t = token t of branch j).
struct TreeSave {
    char* kc;          // [L][Rc][n_kv hd]
    char* vc;          // same shape
    int32_t Tc;        // rows reserved per branch
    size_t layer_bytes;
};

int32_t forward_tree(const atts_model* m, ScoreShape s, int32_t row0, atts_prefix* pre, bool save, bool score,
                     const int32_t* prefix_ids, const int32_t* draft_ids, const int32_t* draft_lens, int32_t score_mode,
                     float* token_logprobs, float* scores, void* workspace, hipStream_t st, const TreeSave* tree = nullptr) {
    const atts_model_desc& d = m->desc;
    const Workspace ws = carve(d, s);
    char* base = static_cast<char*>(workspace);
    float* h = reinterpret_cast<float*>(base + ws.h);
    char* xn = base + ws.xn;
    char* qkv = base + ws.qkv;
    char* vt = attention_uses_vt(d.dtype, d.head_dim) ? base + ws.vt : nullptr;
    char* ao = base + ws.ao;
    char* act = base + ws.act;
    float2* rope = reinterpret_cast<float2*>(base + ws.rope);
    void* xs = base + ws.xs;
    int32_t* targets = reinterpret_cast<int32_t*>(base + ws.targets);
    uint8_t* valid = reinterpret_cast<uint8_t*>(base + ws.valid);
    float2* partials = reinterpret_cast<float2*>(base + ws.partials);
    float* zt = reinterpret_cast<float*>(base + ws.zt);
    float* lp = reinterpret_cast<float*>(base + ws.lp);

    const size_t es = dtype_size(d.dtype);
    const int R = s.R(), B = s.B(), M = R - row0;       // M rows go through the projections
    const int qd = d.n_q_heads * d.head_dim, kvd = d.n_kv_heads * d.head_dim;
    const int qkv_out = (d.n_q_heads + 2 * d.n_kv_heads) * d.head_dim;
    const bool padded = pads_rows(d);
    // the fused epilogue writes 4 transposed-V columns per store: the first computed row must keep them aligned
    // (a continuation call wants the value rows in the qkv buffer: the unfused path leaves them there)
    const bool fuse_rope = vt != nullptr && !tree && row0 % 4 == 0 && qkv_rope_fusable(d.dtype, M, qkv_out, d.d_model, d.head_dim, padded);
    float* h0 = h + (size_t)row0 * d.d_model;
    // few rows: projections with a narrow output cut their K range over the chip (one partial result per slice in
    // kpart); the consumers add the slices in order: the QKV finish (RoPE / V transpose), and the residual update, which
    // also applies the RMSNorm that follows it
    float* kpart = reinterpret_cast<float*>(base + ws.kpart);
    SplitPlan plan = split_plan(d, M);
    if (!fuse_rope) plan.qkv = 1;
    const bool split_qkv = plan.qkv > 1;

    {
        StageTimer t_(ATTS_STAGE_EMBED, st);
        ATTS_TRY(launch_embed(d.dtype, m->tok_embed, d.vocab, d.d_model, prefix_ids, draft_ids, draft_lens, s, row0, h, m->err_flag, st));
        ATTS_TRY(launch_rope_table(rope, s, row0, d.head_dim, d.rope_theta, st));
        // the fused QKV epilogue writes only the R real columns of V^T
        if (fuse_rope) ATTS_TRY(launch_zero_vt_tail(d.dtype, vt, (int64_t)kvd, R, ws.ldv, st));
    }
    char* xn0 = xn + (size_t)row0 * d.d_model * es;
    bool xn_ready = false;      // xn already holds the attention norm of this layer (written with the previous residual update)
    for (int l = 0; l < d.n_layers; ++l) {
        if (!xn_ready) {
            StageTimer t_(ATTS_STAGE_NORM, st);
            ATTS_TRY(launch_rmsnorm(d.dtype, h0, m->attn_norm[l], d.rms_eps, M, d.d_model, xn0, st));
        }
        GemmArgs g{};
        g.a = xn + (size_t)row0 * d.d_model * es; g.w = m->wqkv[l]; g.out = qkv + (size_t)row0 * qkv_out * es;
        g.M = M; g.N = qkv_out; g.Kd = d.d_model;
        g.lda = d.d_model; g.ldw = d.d_model; g.ldc = qkv_out; g.a_rows_padded = padded;
        if (split_qkv) {
            g.out = kpart; g.n_slices = plan.qkv;
            StageTimer t_(ATTS_STAGE_GEMM_QKV, st);
            ATTS_TRY(launch_gemm(d.dtype, EPI_PARTIAL_F32, g, st));
            ATTS_TRY(launch_qkv_finish(d.dtype, kpart, plan.qkv, (int64_t)M * qkv_out, rope + (size_t)row0 * (d.head_dim / 2), M,
                                       d.n_q_heads, d.n_kv_heads, d.head_dim, qkv + (size_t)row0 * qkv_out * es,
                                       vt + (size_t)row0 * es, ws.ldv, st));
        } else if (fuse_rope) {
            // QKV projection with RoPE and the V transpose applied to the accumulators
            g.rope = rope + (size_t)row0 * (d.head_dim / 2); g.vt = vt + (size_t)row0 * es; g.ldv = ws.ldv;
            g.n_rot_heads = d.n_q_heads + d.n_kv_heads;
            StageTimer t_(ATTS_STAGE_GEMM_QKV, st);
            ATTS_TRY(launch_gemm(d.dtype, EPI_QKV_ROPE, g, st));
        } else {
            {
                StageTimer t_(ATTS_STAGE_GEMM_QKV, st);
                ATTS_TRY(launch_gemm(d.dtype, EPI_STORE_ACT, g, st));
            }
            StageTimer t_(ATTS_STAGE_ROPE, st);
            ATTS_TRY(launch_rope_split(d.dtype, qkv, rope, s, row0, d.n_q_heads, d.n_kv_heads, d.head_dim, vt, ws.ldv, st));
        }
        if (pre) {
            // keys / values of the cached prefix rows into place; in save mode the new rows' into the cache
            StageTimer t_(ATTS_STAGE_ROPE, st);
            char* kc = pre->k_cache + (size_t)l * pre->capacity * kvd * es;
            char* wk = qkv + (size_t)qd * es;                                   // key columns of workspace row 0
            ATTS_TRY(launch_copy2d(d.dtype, kc, kvd, wk, qkv_out, row0, kvd, st));
            if (save) ATTS_TRY(launch_copy2d(d.dtype, wk + (size_t)row0 * qkv_out * es, qkv_out, kc + (size_t)row0 * kvd * es, kvd, M, kvd, st));
            if (pre->uses_vt) {
                char* vc = pre->v_cache + (size_t)l * kvd * pre->cap_ld * es;
                ATTS_TRY(launch_copy2d(d.dtype, vc, pre->cap_ld, vt, ws.ldv, kvd, row0, st));
                if (save) ATTS_TRY(launch_copy2d(d.dtype, vt + (size_t)row0 * es, ws.ldv, vc + (size_t)row0 * es, pre->cap_ld, kvd, M, st));
            } else {
                char* vc = pre->v_cache + (size_t)l * pre->capacity * kvd * es;
                char* wv = qkv + (size_t)(qd + kvd) * es;
                ATTS_TRY(launch_copy2d(d.dtype, vc, kvd, wv, qkv_out, row0, kvd, st));
                if (save) ATTS_TRY(launch_copy2d(d.dtype, wv + (size_t)row0 * qkv_out * es, qkv_out, vc + (size_t)row0 * kvd * es, kvd, M, kvd, st));
            }
        }
        if (tree) {
            // keys / values of the whole tree as rows into the continuation cache of this layer (pre != nullptr)
            char* kc = tree->kc + (size_t)l * tree->layer_bytes;
            char* vc = tree->vc + (size_t)l * tree->layer_bytes;
            ATTS_TRY(launch_copy2d(d.dtype, pre->k_cache + (size_t)l * pre->capacity * kvd * es, kvd, kc, kvd, row0, kvd, st));
            if (pre->uses_vt)
                ATTS_TRY(launch_transpose_to_rows(d.dtype, pre->v_cache + (size_t)l * kvd * pre->cap_ld * es, pre->cap_ld, vc, kvd, row0, kvd, st));
            else
                ATTS_TRY(launch_copy2d(d.dtype, pre->v_cache + (size_t)l * pre->capacity * kvd * es, kvd, vc, kvd, row0, kvd, st));
            ATTS_TRY(launch_tree_rows_to_cache(d.dtype, qkv + (size_t)qd * es, qkv_out, kc, kvd, s.P, s.T, tree->Tc, M, kvd, st));
            ATTS_TRY(launch_tree_rows_to_cache(d.dtype, qkv + (size_t)(qd + kvd) * es, qkv_out, vc, kvd, s.P, s.T, tree->Tc, M, kvd, st));
        }
        {
            StageTimer t_(ATTS_STAGE_ATTENTION, st);
            ATTS_TRY(launch_attention(d.dtype, qkv, vt, ws.ldv, ao, s, row0, d.n_q_heads, d.n_kv_heads, d.head_dim, st));
        }
        g = GemmArgs{};
        g.a = ao + (size_t)row0 * qd * es; g.w = m->wo[l]; g.out = h0; g.M = M; g.N = d.d_model; g.Kd = qd;
        g.lda = qd; g.ldw = qd; g.ldc = d.d_model; g.a_rows_padded = padded;
        if (plan.o > 1) {
            g.out = kpart; g.n_slices = plan.o;
            {
                StageTimer t_(ATTS_STAGE_GEMM_O, st);
                ATTS_TRY(launch_gemm(d.dtype, EPI_PARTIAL_F32, g, st));
            }
            StageTimer t_(ATTS_STAGE_NORM, st);
            ATTS_TRY(launch_resid_norm(d.dtype, h0, kpart, plan.o, (int64_t)M * d.d_model, m->ffn_norm[l], d.rms_eps, M, d.d_model, xn0, st));
        } else {
            {
                StageTimer t_(ATTS_STAGE_GEMM_O, st);
                ATTS_TRY(launch_gemm(d.dtype, EPI_RESID_F32, g, st));
            }
            StageTimer t_(ATTS_STAGE_NORM, st);
            ATTS_TRY(launch_rmsnorm(d.dtype, h0, m->ffn_norm[l], d.rms_eps, M, d.d_model, xn0, st));
        }
        g = GemmArgs{};
        g.a = xn0; g.w = m->w_gate_up[l]; g.out = act + (size_t)row0 * d.d_ffn * es;
        g.M = M; g.N = d.d_ffn; g.Kd = d.d_model;
        g.lda = d.d_model; g.ldw = d.d_model; g.ldc = d.d_ffn; g.a_rows_padded = padded;
        {
            StageTimer t_(ATTS_STAGE_GEMM_GATE_UP, st);
            ATTS_TRY(launch_gemm(d.dtype, EPI_SWIGLU, g, st));
        }
        g = GemmArgs{};
        g.a = act + (size_t)row0 * d.d_ffn * es; g.w = m->w_down[l]; g.out = h0; g.M = M; g.N = d.d_model; g.Kd = d.d_ffn;
        g.lda = d.d_ffn; g.ldw = d.d_ffn; g.ldc = d.d_model; g.a_rows_padded = padded;
        if (plan.down > 1) {
            g.out = kpart; g.n_slices = plan.down;
            {
                StageTimer t_(ATTS_STAGE_GEMM_DOWN, st);
                ATTS_TRY(launch_gemm(d.dtype, EPI_PARTIAL_F32, g, st));
            }
            // with the next layer's attention norm (none after the last layer: the final norm runs on the scoring rows only)
            xn_ready = l + 1 < d.n_layers;
            StageTimer t_(ATTS_STAGE_NORM, st);
            ATTS_TRY(launch_resid_norm(d.dtype, h0, kpart, plan.down, (int64_t)M * d.d_model, xn_ready ? m->attn_norm[l + 1] : nullptr,
                                       d.rms_eps, M, d.d_model, xn0, st));
        } else {
            StageTimer t_(ATTS_STAGE_GEMM_DOWN, st);
            ATTS_TRY(launch_gemm(d.dtype, EPI_RESID_F32, g, st));
        }
    }
    if (save) ATTS_HIP_TRY(hipMemcpyAsync(pre->h_last, h + (size_t)(R - 1) * d.d_model, d.d_model * sizeof(float), hipMemcpyDeviceToDevice, st));
    if (!score) return ATTS_OK;
    // the first token of every draft is predicted from the last prefix row
    if (pre && row0 > 0) ATTS_HIP_TRY(hipMemcpyAsync(h + (size_t)(s.P - 1) * d.d_model, pre->h_last, d.d_model * sizeof(float), hipMemcpyDeviceToDevice, st));
    {
        StageTimer t_(ATTS_STAGE_GATHER_NORM, st);
        ATTS_TRY(launch_gather_norm(d.dtype, h, m->final_norm, d.rms_eps, d.d_model, draft_ids, draft_lens, d.vocab, s, xs,
                                    targets, valid, st));
    }
    GemmArgs g{};
    g.a = xs; g.w = m->lm_head; g.out = nullptr; g.M = B; g.N = d.vocab; g.Kd = d.d_model;
    g.lda = d.d_model; g.ldw = d.d_model; g.ldc = 0; g.a_rows_padded = padded;
    g.targets = targets; g.partials = partials; g.target_logit = zt; g.n_part = ws.n_part;
    {
        StageTimer t_(ATTS_STAGE_LMHEAD, st);
        ATTS_TRY(launch_gemm(d.dtype, EPI_LMHEAD, g, st));
    }
    {
        StageTimer t_(ATTS_STAGE_REDUCE, st);
        ATTS_TRY(launch_lmhead_combine(partials, zt, B, ws.n_part, valid, lp, st));
        ATTS_TRY(launch_score_reduce(lp, draft_lens, s.K, s.T, score_mode, token_logprobs, scores, st));
    }
    return ATTS_OK;
}

// Everything about a forward pass over the token tree that the host can refuse: the attention kernel's context limit
// and the workspace.  Called before the first launch of every entry point that runs forward_tree.
int32_t check_workspace(const char* fn, const atts_model_desc& d, ScoreShape s, void* workspace, size_t workspace_bytes) {
    ATTS_TRY(attention_context_check(fn, d.dtype, d.head_dim, s.P, s.T));
    const Workspace ws = carve(d, s);
    if (!workspace || ((uintptr_t)workspace & 255)) return fail(ATTS_ERR_WORKSPACE, "%s: workspace is NULL or not 256-byte aligned", fn);
    if (workspace_bytes < ws.total) return fail(ATTS_ERR_WORKSPACE, "%s: workspace has %zu bytes, %zu needed", fn, workspace_bytes, ws.total);
    return ATTS_OK;
}

}  // namespace
}  // namespace atts

extern "C" {

int32_t atts_score_drafts(const atts_model* m, const int32_t* prefix_ids, int32_t P, const int32_t* draft_ids,
                          const int32_t* draft_lens, int32_t K, int32_t T_max, int32_t score_mode, float* token_logprobs,
                          float* scores, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!m) return fail(ATTS_ERR_INVALID_ARG, "atts_score_drafts: NULL model");
    if (!prefix_ids || !draft_ids || !scores) return fail(ATTS_ERR_INVALID_ARG, "atts_score_drafts: NULL prefix_ids / draft_ids / scores");
    ATTS_TRY(check_score_shape("atts_score_drafts", P, K, T_max));
    if (score_mode != ATTS_SCORE_MEAN_NLL && score_mode != ATTS_SCORE_SUM_NLL)
        return fail(ATTS_ERR_INVALID_ARG, "atts_score_drafts: unknown score_mode %d", score_mode);
    const ScoreShape s{P, K, T_max};
    ATTS_TRY(check_workspace("atts_score_drafts", m->desc, s, workspace, workspace_bytes));
    return forward_tree(m, s, 0, nullptr, false, true, prefix_ids, draft_ids, draft_lens, score_mode, token_logprobs, scores,
                        workspace, static_cast<hipStream_t>(hip_stream));
}

// ---------------------------------------------------------------------------- prefix handle

int32_t atts_prefix_create(const atts_model* m, int32_t capacity, atts_prefix** out) {
    if (!out) return fail(ATTS_ERR_INVALID_ARG, "atts_prefix_create: out is NULL");
    *out = nullptr;
    if (!m) return fail(ATTS_ERR_INVALID_ARG, "atts_prefix_create: NULL model");
    if (capacity < 1 || capacity > (1 << 20)) return fail(ATTS_ERR_INVALID_ARG, "atts_prefix_create: capacity %d outside [1, 1048576]", capacity);
    const atts_model_desc& d = m->desc;
    atts_prefix* p = new (std::nothrow) atts_prefix();
    if (!p) return fail(ATTS_ERR_HIP, "atts_prefix_create: out of host memory");
    p->model = m;
    p->capacity = capacity;
    p->P = 0;
    p->cap_ld = (int64_t)align_up((size_t)capacity, 64);
    p->uses_vt = attention_uses_vt(d.dtype, d.head_dim);
    p->k_cache = p->v_cache = nullptr;
    p->h_last = nullptr;
    const size_t es = dtype_size(d.dtype), kvd = (size_t)d.n_kv_heads * d.head_dim, L = (size_t)(d.n_layers > 0 ? d.n_layers : 1);
    const size_t kb = L * capacity * kvd * es, vb = L * kvd * (p->uses_vt ? (size_t)p->cap_ld : (size_t)capacity) * es;
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&p->k_cache), kb);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&p->v_cache), vb);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&p->h_last), (size_t)d.d_model * sizeof(float));
    if (e != hipSuccess) {
        (void)hipFree(p->k_cache);
        (void)hipFree(p->v_cache);
        (void)hipFree(p->h_last);
        delete p;
        return fail(ATTS_ERR_HIP, "atts_prefix_create: device allocation of %zu bytes failed: %s", kb + vb, hipGetErrorString(e));
    }
    *out = p;
    return ATTS_OK;
}

int32_t atts_prefix_destroy(atts_prefix* p) {
    if (!p) return ATTS_OK;
    (void)hipFree(p->k_cache);
    (void)hipFree(p->v_cache);
    (void)hipFree(p->h_last);
    delete p;
    return ATTS_OK;
}

int32_t atts_prefix_length(const atts_prefix* p, int32_t* out_rows) {
    if (!p || !out_rows) return fail(ATTS_ERR_INVALID_ARG, "atts_prefix_length: NULL argument");
    *out_rows = p->P;
    return ATTS_OK;
}

int32_t atts_prefix_reset(atts_prefix* p) {
    if (!p) return fail(ATTS_ERR_INVALID_ARG, "atts_prefix_reset: NULL handle");
    p->P = 0;
    return ATTS_OK;
}

int32_t atts_prefix_extend_workspace_bytes(const atts_prefix* p, int32_t n, size_t* out_bytes) {
    if (!p || !out_bytes) return fail(ATTS_ERR_INVALID_ARG, "atts_prefix_extend_workspace_bytes: NULL argument");
    if (n < 1 || (int64_t)p->P + n > p->capacity)
        return fail(ATTS_ERR_CAPACITY, "atts_prefix_extend_workspace_bytes: %d + %d rows exceed the capacity %d", p->P, n, p->capacity);
    *out_bytes = carve(p->model->desc, ScoreShape{p->P, 1, n}).total;
    return ATTS_OK;
}

int32_t atts_prefix_extend(atts_prefix* p, const int32_t* ids, int32_t n, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!p) return fail(ATTS_ERR_INVALID_ARG, "atts_prefix_extend: NULL handle");
    if (n < 0) return fail(ATTS_ERR_INVALID_ARG, "atts_prefix_extend: n = %d < 0", n);
    if (n == 0) return ATTS_OK;
    if (!ids) return fail(ATTS_ERR_INVALID_ARG, "atts_prefix_extend: ids is NULL");
    if ((int64_t)p->P + n > p->capacity)
        return fail(ATTS_ERR_CAPACITY, "atts_prefix_extend: %d + %d rows exceed the capacity %d", p->P, n, p->capacity);
    const ScoreShape s{p->P, 1, n};
    ATTS_TRY(check_workspace("atts_prefix_extend", p->model->desc, s, workspace, workspace_bytes));
    // the new rows are one "draft" of n tokens after the cached prefix: plain causal continuation
    ATTS_TRY(forward_tree(p->model, s, p->P, p, true, false, nullptr, ids, nullptr, ATTS_SCORE_MEAN_NLL, nullptr, nullptr, workspace,
                          static_cast<hipStream_t>(hip_stream)));
    p->P += n;
    return ATTS_OK;
}

int32_t atts_score_drafts_cached(const atts_prefix* p, const int32_t* draft_ids, const int32_t* draft_lens, int32_t K,
                                 int32_t T_max, int32_t score_mode, float* token_logprobs, float* scores, void* workspace,
                                 size_t workspace_bytes, void* hip_stream) {
    if (!p) return fail(ATTS_ERR_INVALID_ARG, "atts_score_drafts_cached: NULL handle");
    if (p->P < 1) return fail(ATTS_ERR_INVALID_ARG, "atts_score_drafts_cached: the prefix is empty");
    if (!draft_ids || !scores) return fail(ATTS_ERR_INVALID_ARG, "atts_score_drafts_cached: NULL draft_ids / scores");
    ATTS_TRY(check_score_shape("atts_score_drafts_cached", p->P, K, T_max));
    if (score_mode != ATTS_SCORE_MEAN_NLL && score_mode != ATTS_SCORE_SUM_NLL)
        return fail(ATTS_ERR_INVALID_ARG, "atts_score_drafts_cached: unknown score_mode %d", score_mode);
    const ScoreShape s{p->P, K, T_max};
    ATTS_TRY(check_workspace("atts_score_drafts_cached", p->model->desc, s, workspace, workspace_bytes));
    return forward_tree(p->model, s, p->P, const_cast<atts_prefix*>(p), false, true, nullptr, draft_ids, draft_lens, score_mode,
                        token_logprobs, scores, workspace, static_cast<hipStream_t>(hip_stream));
}

// ---------------------------------------------------------------------------- continuation

namespace {
struct ContinueSpace {
    size_t scoring, kc, vc, h, xn, ao, act, xs, kpart, q, logits, argmax, rope, total;
    int32_t Tc;
    size_t layer_bytes;
};

ContinueSpace carve_continue(const atts_model_desc& d, int32_t P, int32_t Kr, int32_t T, int32_t n_new) {
    const size_t es = dtype_size(d.dtype);
    const size_t kvd = (size_t)d.n_kv_heads * d.head_dim, qd = (size_t)d.n_q_heads * d.head_dim;
    const size_t qkv_out = qd + 2 * kvd, L = (size_t)(d.n_layers > 0 ? d.n_layers : 1);
    const size_t rows_a = pads_rows(d) ? align_up((size_t)Kr, 768) : (size_t)Kr;    // A operands of the aligned GEMM
    ContinueSpace c{};
    c.Tc = T + n_new;
    const size_t Rc = (size_t)P + (size_t)Kr * c.Tc;
    c.layer_bytes = align_up(Rc * kvd * es, 256);
    size_t off = align_up(carve(d, ScoreShape{P, Kr, T}).total, 256);
    c.scoring = 0;
    auto take = [&](size_t bytes) {
        size_t at = off;
        off += align_up(bytes, 256);
        return at;
    };
    c.kc = take(L * c.layer_bytes);
    c.vc = take(L * c.layer_bytes);
    c.h = take((size_t)Kr * d.d_model * sizeof(float));
    c.xn = take(rows_a * d.d_model * es);
    c.ao = take(rows_a * qd * es);
    c.act = take(rows_a * (size_t)d.d_ffn * es);
    c.xs = take(rows_a * d.d_model * es);
    // a decoding step's projections with a narrow output: one partial result per K slice (or the one full result)
    {
        SplitPlan sp = split_plan(d, Kr);
        sp.qkv = gemm_partial_slices(d.dtype, Kr, (int32_t)qkv_out, d.d_model, pads_rows(d));
        c.kpart = take(std::max(sp.bytes, (size_t)sp.qkv * Kr * qkv_out * sizeof(float)));
    }
    c.q = take((size_t)Kr * qd * es);
    c.logits = take((size_t)Kr * d.vocab * sizeof(float));
    c.argmax = take(argmax_scratch_bytes(Kr));
    c.rope = take(((size_t)P + c.Tc) * (d.head_dim / 2) * sizeof(float2));
    c.total = off;
    return c;
}

int32_t check_continue_shape(const char* fn, const atts_prefix* p, int32_t Kr, int32_t T, int32_t n_new) {
    if (!p) return fail(ATTS_ERR_INVALID_ARG, "%s: NULL handle", fn);
    if (p->P < 1) return fail(ATTS_ERR_INVALID_ARG, "%s: the prefix is empty", fn);
    if (Kr < 1 || Kr > 768 || T < 1 || n_new < 1)
        return fail(ATTS_ERR_INVALID_ARG, "%s: need 1 <= K <= 768, T >= 1, n_new >= 1 (K = %d, T = %d, n_new = %d)", fn, Kr, T, n_new);
    return check_score_shape(fn, p->P, Kr, T + n_new);
}
}  // namespace

int32_t atts_continue_workspace_bytes(const atts_prefix* p, int32_t K, int32_t T, int32_t n_new, size_t* out_bytes) {
    if (!out_bytes) return fail(ATTS_ERR_INVALID_ARG, "atts_continue_workspace_bytes: out_bytes is NULL");
    ATTS_TRY(check_continue_shape("atts_continue_workspace_bytes", p, K, T, n_new));
    *out_bytes = carve_continue(p->model->desc, p->P, K, T, n_new).total;
    return ATTS_OK;
}

namespace {
// uniforms == nullptr: greedy; else token t of candidate k is drawn with uniforms[k n_new + t] at inv_temp
int32_t continue_tokens(const char* fn, const atts_prefix* p, const int32_t* draft_ids, const int32_t* draft_lens, int32_t K,
                        int32_t T, int32_t n_new, int32_t eos_id, const float* uniforms, float inv_temp, int32_t* out_ids,
                        void* workspace, size_t workspace_bytes, void* hip_stream) {
    ATTS_TRY(check_continue_shape(fn, p, K, T, n_new));
    if (!draft_ids || !out_ids) return fail(ATTS_ERR_INVALID_ARG, "%s: NULL draft_ids / out_ids", fn);
    const atts_model* m = p->model;
    const atts_model_desc& d = m->desc;
    const int32_t P = p->P;
    ATTS_TRY(attention_context_check(fn, d.dtype, d.head_dim, P, T));
    ATTS_TRY(decode_context_check(fn, d.dtype, d.head_dim, (int64_t)P + T + n_new));
    const ContinueSpace cs = carve_continue(d, P, K, T, n_new);
    if (!workspace || ((uintptr_t)workspace & 255)) return fail(ATTS_ERR_WORKSPACE, "%s: workspace is NULL or not 256-byte aligned", fn);
    if (workspace_bytes < cs.total) return fail(ATTS_ERR_WORKSPACE, "%s: workspace has %zu bytes, %zu needed", fn, workspace_bytes, cs.total);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    char* base = static_cast<char*>(workspace);
    const int qd = d.n_q_heads * d.head_dim, kvd = d.n_kv_heads * d.head_dim, qkv_out = qd + 2 * kvd;
    const bool padded = pads_rows(d);
    const ScoreShape s{P, K, T};

    // 1. the drafts through the model against the cached prefix; keys / values of the whole tree kept per layer
    TreeSave tree{base + cs.kc, base + cs.vc, cs.Tc, cs.layer_bytes};
    ATTS_TRY(forward_tree(m, s, P, const_cast<atts_prefix*>(p), false, false, nullptr, draft_ids, draft_lens, ATTS_SCORE_MEAN_NLL,
                          nullptr, nullptr, workspace, st, &tree));
    const float* h_tree = reinterpret_cast<const float*>(base + carve(d, s).h);

    float* h = reinterpret_cast<float*>(base + cs.h);
    char* xn = base + cs.xn;
    char* ao = base + cs.ao;
    char* act = base + cs.act;
    char* xs = base + cs.xs;
    float* kpart = reinterpret_cast<float*>(base + cs.kpart);
    char* q = base + cs.q;
    float* logits = reinterpret_cast<float*>(base + cs.logits);
    float2* rope = reinterpret_cast<float2*>(base + cs.rope);
    // (cos, sin) rows of the positions new tokens can take: P + 1 ... P + T + n_new - 1 (indexed by absolute position)
    ATTS_TRY(launch_rope_table(rope, ScoreShape{P, 1, cs.Tc}, P, d.head_dim, d.rope_theta, st));
    // the projections of a step that have a narrow output cut their K range over the chip, one partial result per slice
    SplitPlan plan = split_plan(d, K);
    plan.qkv = gemm_partial_slices(d.dtype, K, qkv_out, d.d_model, padded);     // the QKV sums always pass through fp32 here

    auto next_token = [&](int t) -> int32_t {     // xs holds the normalised last hidden states: logits, arg max -> out_ids[:, t]
        GemmArgs g{};
        g.a = xs; g.w = m->lm_head; g.out = logits; g.M = K; g.N = d.vocab; g.Kd = d.d_model;
        g.lda = d.d_model; g.ldw = d.d_model; g.ldc = d.vocab; g.a_rows_padded = padded;
        ATTS_TRY(launch_gemm(d.dtype, EPI_STORE_F32, g, st));
        if (uniforms)
            return launch_sample_rows(logits, d.vocab, d.vocab, K, inv_temp, uniforms + t, base + cs.argmax, out_ids + t, n_new, eos_id,
                                      t > 0, st);
        return launch_argmax_rows(logits, d.vocab, d.vocab, K, base + cs.argmax, out_ids + t, n_new, eos_id, t > 0, st);
    };

    // 2. token 0 follows from the last draft row of every branch: row P + j T + len_j - 1 of the tree
    ATTS_TRY(launch_norm_strided_rows(d.dtype, h_tree, m->final_norm, d.rms_eps, d.d_model, (int64_t)P - 1, T,
                                      BranchPos{draft_lens, T, 0}, K, xs, st));
    ATTS_TRY(next_token(0));

    // 3. one row per branch and step: token t - 1 goes in at branch position len_j + t - 1 and predicts token t
    for (int t = 1; t < n_new; ++t) {
        const BranchPos pos{draft_lens, T, t - 1};
        ATTS_TRY(launch_embed_rows(d.dtype, m->tok_embed, d.vocab, d.d_model, out_ids + (t - 1), n_new, K, h, m->err_flag, st));
        bool xn_ready = false;
        for (int l = 0; l < d.n_layers; ++l) {
            char* kc = tree.kc + (size_t)l * tree.layer_bytes;
            char* vc = tree.vc + (size_t)l * tree.layer_bytes;
            if (!xn_ready) ATTS_TRY(launch_rmsnorm(d.dtype, h, m->attn_norm[l], d.rms_eps, K, d.d_model, xn, st));
            GemmArgs g{};
            g.a = xn; g.w = m->wqkv[l]; g.out = kpart; g.M = K; g.N = qkv_out; g.Kd = d.d_model;
            g.lda = d.d_model; g.ldw = d.d_model; g.ldc = qkv_out; g.a_rows_padded = padded;
            g.n_slices = plan.qkv;
            ATTS_TRY(launch_gemm(d.dtype, plan.qkv > 1 ? EPI_PARTIAL_F32 : EPI_STORE_F32, g, st));
            ATTS_TRY(launch_decode_qkv_finish(d.dtype, kpart, plan.qkv, (int64_t)K * qkv_out, rope, K, d.n_q_heads, d.n_kv_heads,
                                              d.head_dim, P, cs.Tc, pos, q, kc, vc, st));
            ATTS_TRY(launch_attn_decode(d.dtype, q, kc, vc, ao, K, P, cs.Tc, pos, d.n_q_heads, d.n_kv_heads, d.head_dim, st));
            g = GemmArgs{};
            g.a = ao; g.w = m->wo[l]; g.out = h; g.M = K; g.N = d.d_model; g.Kd = qd;
            g.lda = qd; g.ldw = qd; g.ldc = d.d_model; g.a_rows_padded = padded;
            if (plan.o > 1) {
                g.out = kpart; g.n_slices = plan.o;
                ATTS_TRY(launch_gemm(d.dtype, EPI_PARTIAL_F32, g, st));
                ATTS_TRY(launch_resid_norm(d.dtype, h, kpart, plan.o, (int64_t)K * d.d_model, m->ffn_norm[l], d.rms_eps, K, d.d_model, xn, st));
            } else {
                ATTS_TRY(launch_gemm(d.dtype, EPI_RESID_F32, g, st));
                ATTS_TRY(launch_rmsnorm(d.dtype, h, m->ffn_norm[l], d.rms_eps, K, d.d_model, xn, st));
            }
            g = GemmArgs{};
            g.a = xn; g.w = m->w_gate_up[l]; g.out = act; g.M = K; g.N = d.d_ffn; g.Kd = d.d_model;
            g.lda = d.d_model; g.ldw = d.d_model; g.ldc = d.d_ffn; g.a_rows_padded = padded;
            ATTS_TRY(launch_gemm(d.dtype, EPI_SWIGLU, g, st));
            g = GemmArgs{};
            g.a = act; g.w = m->w_down[l]; g.out = h; g.M = K; g.N = d.d_model; g.Kd = d.d_ffn;
            g.lda = d.d_ffn; g.ldw = d.d_ffn; g.ldc = d.d_model; g.a_rows_padded = padded;
            if (plan.down > 1) {
                g.out = kpart; g.n_slices = plan.down;
                ATTS_TRY(launch_gemm(d.dtype, EPI_PARTIAL_F32, g, st));
                xn_ready = l + 1 < d.n_layers;
                ATTS_TRY(launch_resid_norm(d.dtype, h, kpart, plan.down, (int64_t)K * d.d_model, xn_ready ? m->attn_norm[l + 1] : nullptr,
                                           d.rms_eps, K, d.d_model, xn, st));
            } else {
                ATTS_TRY(launch_gemm(d.dtype, EPI_RESID_F32, g, st));
                xn_ready = false;
            }
        }
        ATTS_TRY(launch_norm_strided_rows(d.dtype, h, m->final_norm, d.rms_eps, d.d_model, 0, 1, BranchPos{nullptr, 0, 0}, K, xs, st));
        ATTS_TRY(next_token(t));
    }
    return ATTS_OK;
}
}  // namespace

int32_t atts_continue_greedy(const atts_prefix* p, const int32_t* draft_ids, const int32_t* draft_lens, int32_t K, int32_t T,
                             int32_t n_new, int32_t eos_id, int32_t* out_ids, void* workspace, size_t workspace_bytes,
                             void* hip_stream) {
    return continue_tokens("atts_continue_greedy", p, draft_ids, draft_lens, K, T, n_new, eos_id, nullptr, 1.f, out_ids, workspace,
                           workspace_bytes, hip_stream);
}

int32_t atts_continue_sample(const atts_prefix* p, const int32_t* draft_ids, const int32_t* draft_lens, int32_t K, int32_t T,
                             int32_t n_new, int32_t eos_id, float temperature, const float* uniforms, int32_t* out_ids,
                             void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!(temperature > 0.f) || !(temperature < INFINITY))
        return fail(ATTS_ERR_INVALID_ARG, "atts_continue_sample: temperature must be positive and finite");
    if (!uniforms) return fail(ATTS_ERR_INVALID_ARG, "atts_continue_sample: uniforms is NULL");
    return continue_tokens("atts_continue_sample", p, draft_ids, draft_lens, K, T, n_new, eos_id, uniforms, 1.f / temperature, out_ids,
                           workspace, workspace_bytes, hip_stream);
}

int32_t atts_model_check(const atts_model* m, void* hip_stream, int32_t* host_flag) {
    if (!m || !host_flag) return fail(ATTS_ERR_INVALID_ARG, "atts_model_check: NULL argument");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    ATTS_HIP_TRY(hipMemcpyAsync(host_flag, m->err_flag, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    ATTS_HIP_TRY(hipStreamSynchronize(st));
    ATTS_HIP_TRY(hipMemsetAsync(m->err_flag, 0, sizeof(int32_t), st));
    ATTS_HIP_TRY(hipStreamSynchronize(st));
    return ATTS_OK;
}

// ---------------------------------------------------------------------------- stage timing

int32_t atts_profile_enable(int32_t on) {
    prof_clear();
    g_prof_on = on != 0;
    return ATTS_OK;
}

int32_t atts_profile_read(int32_t stage, double* total_ms, int64_t* launches) {
    if (stage < 0 || stage >= ATTS_STAGE_COUNT) return fail(ATTS_ERR_INVALID_ARG, "atts_profile_read: unknown stage %d", stage);
    double ms = 0.0;
    int64_t n = 0;
    for (const auto& r : g_prof) {
        if (r.stage != stage) continue;
        ATTS_HIP_TRY(hipEventSynchronize(r.stop));
        float t = 0.f;
        ATTS_HIP_TRY(hipEventElapsedTime(&t, r.start, r.stop));
        ms += t;
        ++n;
    }
    if (total_ms) *total_ms = ms;
    if (launches) *launches = n;
    return ATTS_OK;
}

// ---------------------------------------------------------------------------- stand-alone stages

int32_t atts_lmhead_workspace_bytes(int32_t B, int32_t V, size_t* out_bytes) {
    if (!out_bytes || B < 1 || V < 1) return fail(ATTS_ERR_INVALID_ARG, "atts_lmhead_workspace_bytes: bad argument");
    // sized for the finest column split any dtype / inner dimension takes
    *out_bytes = align_up((size_t)B * lmhead_max_partials(V) * sizeof(float2), 256) + align_up((size_t)B * sizeof(float), 256);
    return ATTS_OK;
}

}  // extern "C"

namespace {
// Scratch of atts_lmhead_logprobs_static: one copy per GPU (each device that loads this code object holds its own, at
// its own address, until the process ends).  In host code the array's name is only a handle for hipGetSymbolAddress:
// kernels are given the address that call returns, looked up once per device with that device current.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int32_t static_scratch_ptr(void** out) {
    int dev = -1;
    ATTS_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(ATTS_ERR_HIP, "static scratch: device index %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        ATTS_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(ATTS_ERR_HIP, "static scratch: hipGetSymbolAddress returned a null address");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return ATTS_OK;
}

// The fused LM head on a scratch area of lmhead_workspace_bytes(B, V) bytes: per-row (max, sum-exp) partials, then the
// target logits.  Shared by the two entry points below.
int32_t lmhead_on_scratch(int32_t dtype, const void* x, const void* w, const int32_t* targets, int32_t B, int32_t d,
                          int32_t V, float* logprobs, void* scratch_area, hipStream_t st) {
    const int n_part = lmhead_num_partials(dtype, B, V, d, false);
    float2* partials = static_cast<float2*>(scratch_area);
    float* zt = reinterpret_cast<float*>(static_cast<char*>(scratch_area) + align_up((size_t)B * lmhead_max_partials(V) * sizeof(float2), 256));
    GemmArgs g{};
    g.a = x; g.w = w; g.M = B; g.N = V; g.Kd = d; g.lda = d; g.ldw = d;
    g.targets = targets; g.partials = partials; g.target_logit = zt; g.n_part = n_part;
    ATTS_TRY(launch_gemm(dtype, EPI_LMHEAD, g, st));
    return launch_lmhead_combine(partials, zt, B, n_part, nullptr, logprobs, st);
}

int32_t check_lmhead_args(const char* fn, int32_t dtype, const void* x, const void* w, const int32_t* targets, int32_t B, int32_t d,
                          int32_t V, const float* logprobs) {
    if (dtype != ATTS_DTYPE_F32 && dtype != ATTS_DTYPE_BF16) return fail(ATTS_ERR_INVALID_ARG, "%s: unknown dtype %d", fn, dtype);
    if (!x || !w || !targets || !logprobs) return fail(ATTS_ERR_INVALID_ARG, "%s: NULL argument", fn);
    if (B < 1 || d < 1 || V < 1) return fail(ATTS_ERR_INVALID_ARG, "%s: B, d, V must be >= 1", fn);
    return ATTS_OK;
}
}  // namespace

extern "C" {

int32_t atts_lmhead_logprobs(int32_t dtype, const void* x, const void* w, const int32_t* targets, int32_t B, int32_t d, int32_t V,
                             float* logprobs, void* workspace, size_t workspace_bytes, void* hip_stream) {
    ATTS_TRY(check_lmhead_args("atts_lmhead_logprobs", dtype, x, w, targets, B, d, V, logprobs));
    size_t need = 0;
    ATTS_TRY(atts_lmhead_workspace_bytes(B, V, &need));
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < need)
        return fail(ATTS_ERR_WORKSPACE, "atts_lmhead_logprobs: workspace NULL, misaligned or smaller than %zu bytes", need);
    return lmhead_on_scratch(dtype, x, w, targets, B, d, V, logprobs, workspace, static_cast<hipStream_t>(hip_stream));
}

// The same stage for callers that cannot allocate: its scratch is the file-scope device array below.
int32_t atts_lmhead_logprobs_static(int32_t dtype, const void* x, const void* w, const int32_t* targets, int32_t B, int32_t d,
                                    int32_t V, float* logprobs, void* hip_stream) {
    ATTS_TRY(check_lmhead_args("atts_lmhead_logprobs_static", dtype, x, w, targets, B, d, V, logprobs));
    size_t need = 0;
    ATTS_TRY(atts_lmhead_workspace_bytes(B, V, &need));
    if (need > kStaticScratchBytes)
        return fail(ATTS_ERR_WORKSPACE, "atts_lmhead_logprobs_static: B = %d rows of a %d-token vocabulary need %zu bytes of scratch, "
                    "the static area holds %zu", B, V, need, kStaticScratchBytes);
    void* area = nullptr;
    ATTS_TRY(static_scratch_ptr(&area));
    return lmhead_on_scratch(dtype, x, w, targets, B, d, V, logprobs, area, static_cast<hipStream_t>(hip_stream));
}

int32_t atts_gemm_nt(int32_t dtype, const void* a, const void* w, float* c, int32_t M, int32_t N, int32_t Kdim, void* hip_stream) {
    if (dtype != ATTS_DTYPE_F32 && dtype != ATTS_DTYPE_BF16) return fail(ATTS_ERR_INVALID_ARG, "atts_gemm_nt: unknown dtype %d", dtype);
    if (!a || !w || !c) return fail(ATTS_ERR_INVALID_ARG, "atts_gemm_nt: NULL argument");
    GemmArgs g{};
    g.a = a; g.w = w; g.out = c; g.M = M; g.N = N; g.Kd = Kdim; g.lda = Kdim; g.ldw = Kdim; g.ldc = N;
    return launch_gemm(dtype, EPI_STORE_F32, g, static_cast<hipStream_t>(hip_stream));
}

int32_t atts_attention_workspace_bytes(int32_t dtype, int32_t R, int32_t n_kv, int32_t hd, size_t* out_bytes) {
    if (!out_bytes || R < 1 || n_kv < 1 || hd < 2) return fail(ATTS_ERR_INVALID_ARG, "atts_attention_workspace_bytes: bad argument");
    *out_bytes = attention_uses_vt(dtype, hd) ? align_up((size_t)n_kv * hd * align_up(R, 64) * dtype_size(dtype), 256) : 0;
    return ATTS_OK;
}

int32_t atts_attention_shared_prefix(int32_t dtype, const void* qkv, void* out, int32_t P, int32_t K, int32_t T, int32_t n_q,
                                     int32_t n_kv, int32_t hd, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (dtype != ATTS_DTYPE_F32 && dtype != ATTS_DTYPE_BF16) return fail(ATTS_ERR_INVALID_ARG, "atts_attention_shared_prefix: unknown dtype %d", dtype);
    if (!qkv || !out) return fail(ATTS_ERR_INVALID_ARG, "atts_attention_shared_prefix: NULL argument");
    if (P < 1 || K < 0 || T < 0 || (K > 0 && T < 1)) return fail(ATTS_ERR_INVALID_ARG, "atts_attention_shared_prefix: need P >= 1 and K = 0 or T >= 1");
    if (n_q < 1 || n_kv < 1 || n_q % n_kv || hd < 2 || hd % 2 || hd > 256 || (hd * dtype_size(dtype)) % 16)
        return fail(ATTS_ERR_SHAPE, "atts_attention_shared_prefix: unsupported head configuration");
    if (K == 0) T = 1;
    ATTS_TRY(check_score_shape("atts_attention_shared_prefix", P, K > 0 ? K : 1, T));
    const ScoreShape s{P, K, T};
    ATTS_TRY(attention_context_check("atts_attention_shared_prefix", dtype, hd, P, T));
    size_t need = 0;
    ATTS_TRY(atts_attention_workspace_bytes(dtype, s.R(), n_kv, hd, &need));
    void* vt = nullptr;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int64_t ldv = (int64_t)align_up(s.R(), 64);
    if (need) {
        if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < need)
            return fail(ATTS_ERR_WORKSPACE, "atts_attention_shared_prefix: workspace NULL, misaligned or smaller than %zu bytes", need);
        vt = workspace;
        ATTS_TRY(launch_transpose_v(dtype, qkv, 0, s.R(), n_q, n_kv, hd, vt, ldv, st));
    }
    return launch_attention(dtype, qkv, vt, ldv, out, s, 0, n_q, n_kv, hd, st);
}

}  // extern "C"
