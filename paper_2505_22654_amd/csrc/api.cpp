// C ABI of the VScan reduction library: argument validation, workspace
// planning and kernel sequencing.  Everything before the first launch is pure
// host code and never touches the HIP runtime, so descriptor errors are
// reported identically with or without a device.
#include "../../include/vscan.h"

#include <math.h>
#include <string.h>

#include <atomic>
#include <mutex>
#include <vector>

#include "fused.hpp"
#include "launch.hpp"
#include "log.hpp"

namespace {

using namespace vscan;

constexpr size_t kAlign = 256;
constexpr size_t kLdsBudget = 160 * 1024;

inline size_t align_up(size_t v) { return (v + kAlign - 1) & ~(kAlign - 1); }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int elem_bytes(int dtype) { return dtype == VSCAN_BF16 ? 2 : 4; }

struct EncoderPlan {
    int N, S, BC, T, W, kw, kg, Kseg, K, U;
    size_t off_head_global, off_head_local, off_lse, off_drop, off_best, off_inv_norm, off_pre_key, off_pre_flag, bytes;
};

int plan_encoder(const vscan_encoder_desc *d, int with_local, EncoderPlan *p) {
    if (!d) return VSCAN_ERR_NULL;
    if (d->struct_size != sizeof(vscan_encoder_desc)) return VSCAN_ERR_VERSION;
    if (d->dtype != VSCAN_F32 && d->dtype != VSCAN_BF16) return VSCAN_ERR_DTYPE;
    if (d->score_mode != VSCAN_SCORE_CLS_ROW && d->score_mode != VSCAN_SCORE_MEAN_RECEIVED)
        return VSCAN_ERR_DTYPE;
    if (d->softmax_domain != VSCAN_KEYS_VISUAL_ONLY && d->softmax_domain != VSCAN_KEYS_ALL)
        return VSCAN_ERR_DTYPE;
    if (d->batch < 0 || d->n_segments < 1 || d->grid_h < 1 || d->grid_w < 1 || d->heads < 1)
        return VSCAN_ERR_SHAPE;
    if (d->has_cls != 0 && d->has_cls != 1) return VSCAN_ERR_SHAPE;
    if (d->score_mode == VSCAN_SCORE_CLS_ROW && !d->has_cls) return VSCAN_ERR_SHAPE;
    if (d->head_dim < 8 || d->head_dim % 8 || d->head_dim > 256) return VSCAN_ERR_SHAPE;
    if (d->feat_dim < 8 || d->feat_dim % 8) return VSCAN_ERR_SHAPE;
    if (d->win_rows < 1 || d->win_cols < 1 || d->win_rows > d->grid_h || d->win_cols > d->grid_w)
        return VSCAN_ERR_SHAPE;
    if ((int64_t)d->grid_h * d->grid_w > (1 << 20)) return VSCAN_ERR_SHAPE;
    if (d->keep_global < 0 || d->keep_local < 0) return VSCAN_ERR_BUDGET;
    const int es = elem_bytes(d->dtype);
    p->N = d->grid_h * d->grid_w;
    p->S = p->N + d->has_cls;
    p->W = d->win_rows * d->win_cols;
    p->kw = d->keep_local / p->W;
    p->kg = d->keep_global + (d->keep_local - p->kw * p->W);
    p->Kseg = d->keep_global + d->keep_local;
    if (p->Kseg < 1 || p->Kseg > p->N) return VSCAN_ERR_BUDGET;
    const int min_window = (d->grid_h / d->win_rows) * (d->grid_w / d->win_cols);
    if (p->kw > min_window) return VSCAN_ERR_BUDGET;
    if ((int64_t)d->batch * d->n_segments > (1 << 24)) return VSCAN_ERR_SHAPE;
    if ((int64_t)d->n_segments * p->N > (1 << 24)) return VSCAN_ERR_SHAPE;
    // (segment, head) pairs index launch grids and 32-bit item counters
    if (d->heads > 1024 || (int64_t)d->batch * d->n_segments * d->heads > (1 << 24))
        return VSCAN_ERR_SHAPE;
    p->BC = d->batch * d->n_segments;
    p->T = d->n_segments * p->N;
    p->K = d->n_segments * p->Kseg;
    p->U = p->T - p->K;
    // limits of the kernels
    if (d->feat_dim * es > 16 * 1024) return VSCAN_ERR_UNSUPPORTED;
    if ((int64_t)p->T * d->feat_dim * es >= ((int64_t)1 << 31)) return VSCAN_ERR_UNSUPPORTED;
    if (d->score_mode == VSCAN_SCORE_MEAN_RECEIVED && d->head_dim * es > 512)
        return VSCAN_ERR_UNSUPPORTED;
    if (encoder_select_lds_bytes(p->N, with_local) > kLdsBudget) return VSCAN_ERR_UNSUPPORTED;
    if ((size_t)(16 + 256 + p->S) * sizeof(float) > kLdsBudget) return VSCAN_ERR_UNSUPPORTED;

    const size_t head = align_up((size_t)p->BC * d->heads * p->N * sizeof(float));
    size_t off = 0;
    p->off_head_global = off;
    off += head;
    p->off_head_local = off;
    if (with_local) off += head;
    p->off_lse = off;
    if (d->score_mode == VSCAN_SCORE_MEAN_RECEIVED) off += head;
    p->off_drop = off;
    off += align_up((size_t)d->batch * p->U * sizeof(int32_t));
    p->off_best = off;
    off += align_up((size_t)d->batch * p->T * sizeof(uint64_t));
    p->off_inv_norm = off;
    off += align_up((size_t)d->batch * p->K * sizeof(float));
    p->off_pre_key = off;
    off += align_up((size_t)p->BC * p->N * sizeof(uint32_t));
    p->off_pre_flag = off;
    off += align_up((size_t)p->BC * p->N);
    p->bytes = off ? off : kAlign;
    return VSCAN_OK;
}

struct LlmPlan {
    int rows, k0, nk, S_out;
    size_t off_part, off_split_e, off_split_stats, bytes;
};

int plan_llm(const vscan_llm_desc *d, LlmPlan *p) {
    if (!d) return VSCAN_ERR_NULL;
    if (d->struct_size != sizeof(vscan_llm_desc)) return VSCAN_ERR_VERSION;
    if (d->dtype != VSCAN_F32 && d->dtype != VSCAN_BF16) return VSCAN_ERR_DTYPE;
    if (d->softmax_domain != VSCAN_KEYS_VISUAL_ONLY && d->softmax_domain != VSCAN_KEYS_ALL)
        return VSCAN_ERR_DTYPE;
    if (d->batch < 0 || d->seq_len < 1 || d->vis_start < 0 || d->vis_len < 1 || d->n_query < 1)
        return VSCAN_ERR_SHAPE;
    if ((int64_t)d->vis_start + d->vis_len + d->n_query > d->seq_len) return VSCAN_ERR_SHAPE;
    if (d->q_heads < 1 || d->kv_heads < 1 || d->q_heads % d->kv_heads) return VSCAN_ERR_SHAPE;
    if (d->q_heads > 1024) return VSCAN_ERR_SHAPE;
    if (d->head_dim < 8 || d->head_dim % 8 || d->head_dim > 256) return VSCAN_ERR_SHAPE;
    if (d->hidden < 8 || d->hidden % 8) return VSCAN_ERR_SHAPE;
    if (d->in_place != 0 && d->in_place != 1) return VSCAN_ERR_SHAPE;
    if ((int64_t)d->batch * d->kv_heads > (1 << 24)) return VSCAN_ERR_SHAPE;
    if (d->keep < 0 || d->keep > d->vis_len) return VSCAN_ERR_BUDGET;
    const int es = elem_bytes(d->dtype);
    p->rows = (d->q_heads / d->kv_heads) * d->n_query;
    p->k0 = d->softmax_domain == VSCAN_KEYS_ALL ? 0 : d->vis_start;
    p->nk = d->softmax_domain == VSCAN_KEYS_ALL ? d->seq_len : d->vis_len;
    p->S_out = d->seq_len - d->vis_len + d->keep;
    if (!llm_score_supported(p->rows, p->nk, d->head_dim * es)) return VSCAN_ERR_UNSUPPORTED;
    if (llm_select_lds_bytes(d->vis_len) > kLdsBudget) return VSCAN_ERR_UNSUPPORTED;
    p->off_part = 0;
    size_t off = align_up((size_t)d->batch * d->kv_heads * d->vis_len * sizeof(float));
    // few items with long key domains are scored chunk by chunk (uniform batches only; the
    // space is part of the plan whenever the shape qualifies)
    const int chunks = llm_score_split_chunks(d->batch, d->kv_heads, p->rows, p->nk, false);
    p->off_split_e = off;
    if (chunks > 0) off += align_up((size_t)d->batch * d->kv_heads * p->rows * d->vis_len * sizeof(float));
    p->off_split_stats = off;
    if (chunks > 0) off += align_up((size_t)d->batch * d->kv_heads * chunks * p->rows * 2 * sizeof(float));
    p->bytes = off ? off : kAlign;
    return VSCAN_OK;
}

// Scratch of the score chain that starts from hidden states and projection weights:
// `seqs` sequences of S rows of `hidden` features, Tq query rows each, nk keys in the domain.
struct FusedScratch {
    int ks_q, ks_l;
    size_t off_cq, off_qpl, off_qtpl, off_cl, end;
};

int plan_fused_scratch(int64_t seqs, int S, int hidden, int q_heads, int kv_heads, int head_dim,
                       int n_query, int nk, int es, size_t base, FusedScratch *f) {
    // 32-bit row offsets inside the kernels (es = bytes per element of hidden states and weights)
    const int64_t lim = (int64_t)1 << 32;
    const int64_t Dh = hidden, N = (int64_t)q_heads * head_dim, R = (int64_t)q_heads * n_query;
    if (seqs * S * Dh * es >= lim || N * Dh * es >= lim || Dh * kv_heads * head_dim * es >= lim ||
        seqs * n_query * N * es >= lim || seqs * R * Dh * es >= lim || seqs * R > (1 << 24) ||
        R > 65535 || seqs > 65535)  // sequences and query rows index the softmax grid
        return VSCAN_ERR_UNSUPPORTED;
    const int M = (int)(seqs * n_query);
    f->ks_q = fused_ksplit((int)N, M, 1, hidden, es);
    f->ks_l = fused_ksplit(nk, (int)R, (int)seqs, hidden, es);
    // q and the hidden-space query: three bf16 planes each for bf16 inputs, the fp32 values
    // themselves for fp32 inputs
    const size_t carried = es == 2 ? (size_t)kFusedQtPlanes * 2 : 4;
    size_t off = base;
    f->off_cq = off;
    off += align_up((size_t)f->ks_q * M * N * sizeof(float));
    f->off_qpl = off;
    off += align_up((size_t)M * N * (es == 2 ? 3 * 2 : 4));
    f->off_qtpl = off;
    off += align_up(carried * seqs * R * Dh);
    f->off_cl = off;
    off += align_up((size_t)f->ks_l * seqs * R * nk * sizeof(float));
    f->end = off;
    return VSCAN_OK;
}

struct FusedPlan {
    int k0, nk, S_out, R;
    FusedScratch f;
    size_t off_part, bytes;
};

int plan_fused(const vscan_llm_desc *d, FusedPlan *p) {
    if (!d) return VSCAN_ERR_NULL;
    if (d->struct_size != sizeof(vscan_llm_desc)) return VSCAN_ERR_VERSION;
    if (d->dtype != VSCAN_F32 && d->dtype != VSCAN_BF16) return VSCAN_ERR_DTYPE;
    if (d->softmax_domain != VSCAN_KEYS_VISUAL_ONLY && d->softmax_domain != VSCAN_KEYS_ALL)
        return VSCAN_ERR_DTYPE;
    if (d->batch < 0 || d->seq_len < 1 || d->vis_start < 0 || d->vis_len < 1 || d->n_query < 1)
        return VSCAN_ERR_SHAPE;
    if ((int64_t)d->vis_start + d->vis_len + d->n_query > d->seq_len) return VSCAN_ERR_SHAPE;
    if (d->q_heads < 1 || d->kv_heads < 1 || d->q_heads % d->kv_heads) return VSCAN_ERR_SHAPE;
    if (d->q_heads > 1024) return VSCAN_ERR_SHAPE;
    if (d->head_dim < 8 || d->head_dim % 8 || d->head_dim > 256) return VSCAN_ERR_SHAPE;
    if (d->hidden < 8 || d->hidden % 8) return VSCAN_ERR_SHAPE;
    if (d->in_place != 0 && d->in_place != 1) return VSCAN_ERR_SHAPE;
    if (d->keep < 0 || d->keep > d->vis_len) return VSCAN_ERR_BUDGET;
    p->k0 = d->softmax_domain == VSCAN_KEYS_ALL ? 0 : d->vis_start;
    p->nk = d->softmax_domain == VSCAN_KEYS_ALL ? d->seq_len : d->vis_len;
    p->S_out = d->seq_len - d->vis_len + d->keep;
    p->R = d->q_heads * d->n_query;
    if (llm_select_lds_bytes(d->vis_len) > kLdsBudget) return VSCAN_ERR_UNSUPPORTED;
    const int rc = plan_fused_scratch(d->batch, d->seq_len, d->hidden, d->q_heads, d->kv_heads,
                                      d->head_dim, d->n_query, p->nk, elem_bytes(d->dtype), 0, &p->f);
    if (rc != VSCAN_OK) return rc;
    p->off_part = p->f.end;
    p->bytes = p->off_part + align_up((size_t)d->batch * d->vis_len * sizeof(float));
    return VSCAN_OK;
}

// Stage 1 scored from hidden states: the ordinary encoder plan, the scratch above behind it.
struct EncoderFusedPlan {
    EncoderPlan e;
    FusedScratch f;
    int k0, nk;
    // mean-attention scoring: W_K with its rows along the output features, then Q and K of
    // every token in fp32 [BC, H, S, dh]
    size_t off_wk, off_qf, off_kf;
    size_t bytes;
};

int plan_encoder_fused(const vscan_encoder_desc *d, int with_local, EncoderFusedPlan *p) {
    const int rc = plan_encoder(d, with_local, &p->e);
    if (rc != VSCAN_OK) return rc;
    const int es = elem_bytes(d->dtype);
    if (d->score_mode == VSCAN_SCORE_MEAN_RECEIVED) {
        // Q and K are projected in fp32 and scored by the fp32 mean-attention kernels
        if (d->head_dim * 4 > 512) return VSCAN_ERR_UNSUPPORTED;
        const int64_t lim = (int64_t)1 << 32;  // 32-bit row offsets inside the projection
        const int64_t feat = (int64_t)d->heads * d->head_dim;
        if ((int64_t)p->e.BC * p->e.S * d->feat_dim * es >= lim || feat * d->feat_dim * es >= lim ||
            (int64_t)p->e.BC * p->e.S >= ((int64_t)1 << 31) / 2)
            return VSCAN_ERR_UNSUPPORTED;
        p->k0 = p->nk = 0;
        p->f = FusedScratch{};
        size_t off = p->e.bytes;
        p->off_wk = off;
        off += align_up((size_t)feat * d->feat_dim * es);
        p->off_qf = off;
        off += align_up((size_t)p->e.BC * feat * p->e.S * sizeof(float));
        p->off_kf = off;
        off += align_up((size_t)p->e.BC * feat * p->e.S * sizeof(float));
        p->bytes = off;
        return VSCAN_OK;
    }
    p->off_wk = p->off_qf = p->off_kf = 0;
    p->k0 = d->softmax_domain == VSCAN_KEYS_ALL ? 0 : 1;
    p->nk = d->softmax_domain == VSCAN_KEYS_ALL ? p->e.S : p->e.N;
    const int rc2 = plan_fused_scratch(p->e.BC, p->e.S, d->feat_dim, d->heads, d->heads,
                                       d->head_dim, 1, p->nk, es, p->e.bytes, &p->f);
    if (rc2 != VSCAN_OK) return rc2;
    p->bytes = p->f.end;
    return VSCAN_OK;
}

inline float resolve_scale(float scale, int head_dim) {
    return scale > 0.f ? scale : 1.0f / sqrtf((float)head_dim);
}

// Logs a failing entry point (debug log only) and passes its status through.
inline int finish(const char *entry, int rc) {
    if (rc != VSCAN_OK) logf("%s -> %d (%s)", entry, rc, vscan_status_string(rc));
    return rc;
}

// ---- per-kernel event timing (measurement aid) ------------------------------
struct ProfRecord {
    const char *name;
    hipEvent_t start, stop;
};
std::mutex g_prof_mutex;
std::vector<ProfRecord> g_prof_records;
std::atomic<bool> g_prof_on{false};  // read by every launch, on any thread

struct ProfScope {
    const char *name;
    hipStream_t stream;
    hipEvent_t start = nullptr, stop = nullptr;
    bool on;
    ProfScope(const char *n, hipStream_t s) : name(n), stream(s), on(g_prof_on.load(std::memory_order_relaxed)) {
        if (!on) return;
        if (hipEventCreate(&start) != hipSuccess || hipEventCreate(&stop) != hipSuccess ||
            hipEventRecord(start, stream) != hipSuccess)
            on = false;
    }
    ~ProfScope() {
        if (!on) return;
        if (hipEventRecord(stop, stream) == hipSuccess) {
            std::lock_guard<std::mutex> lock(g_prof_mutex);
            g_prof_records.push_back({name, start, stop});
        }
    }
};

#define VSCAN_LAUNCH(name, call)                                                  \
    do {                                                                          \
        hipError_t e_;                                                            \
        {                                                                         \
            ProfScope scope_(name, s);                                            \
            e_ = (call);                                                          \
        }                                                                         \
        if (e_ != hipSuccess) {                                                   \
            logf("launch of %s failed: %s", name, hipGetErrorString(e_));         \
            return VSCAN_ERR_HIP;                                                 \
        }                                                                         \
        logf("enqueued %s", name);                                                \
    } while (0)

// The score chain: part[seq][token] = sum over the query rows of their softmax weights.
int enqueue_fused_scores(FusedArgs &fa, const FusedScratch &f, unsigned char *ws, hipStream_t s) {
    fa.c_q = reinterpret_cast<float *>(ws + f.off_cq);
    fa.q_planes = reinterpret_cast<uint16_t *>(ws + f.off_qpl);
    fa.qt_planes = reinterpret_cast<uint16_t *>(ws + f.off_qtpl);
    fa.c_l = reinterpret_cast<float *>(ws + f.off_cl);
    fa.ks_q = f.ks_q;
    fa.ks_l = f.ks_l;
    VSCAN_LAUNCH("fused_q", launch_fused_q(fa, s));
    VSCAN_LAUNCH("fused_split_q", launch_fused_split_q(fa, s));
    VSCAN_LAUNCH("fused_qt", launch_fused_qt(fa, s));
    VSCAN_LAUNCH("fused_logits", launch_fused_logits(fa, s));
    VSCAN_LAUNCH("fused_softmax", launch_fused_softmax(fa, s));
    VSCAN_LAUNCH("fused_colsum", launch_fused_colsum(fa, s));
    return VSCAN_OK;
}

// Selection, assignment and merge of stage 1 from per-head scores in the workspace.
int enqueue_encoder_tail(const vscan_encoder_desc *d, const EncoderPlan &p, bool with_local,
                         int score_heads, float norm, const void *x, int32_t *kept_idx,
                         void *merged, int32_t *assign_out, float *scores_out, unsigned char *ws,
                         hipStream_t s) {
    EncSelectArgs se;
    se.head_global = reinterpret_cast<const float *>(ws + p.off_head_global);
    se.head_local = with_local ? reinterpret_cast<const float *>(ws + p.off_head_local) : nullptr;
    se.B = d->batch;
    se.C = d->n_segments;
    se.H = score_heads;
    se.gh = d->grid_h;
    se.gw = d->grid_w;
    se.wr = d->win_rows;
    se.wc = d->win_cols;
    se.kw = p.kw;
    se.kg = p.kg;
    se.norm = norm;
    se.kept_idx = kept_idx;
    se.drop_idx = reinterpret_cast<int32_t *>(ws + p.off_drop);
    se.best = reinterpret_cast<uint64_t *>(ws + p.off_best);
    se.scores_out = scores_out;
    se.pre_key_ws = reinterpret_cast<uint32_t *>(ws + p.off_pre_key);
    se.pre_flag_ws = reinterpret_cast<uint8_t *>(ws + p.off_pre_flag);
    VSCAN_LAUNCH("encoder_select", launch_encoder_select(se, s));

    MergeArgs ma;
    ma.x = x;
    ma.kept_idx = kept_idx;
    ma.drop_idx = se.drop_idx;
    ma.best = se.best;
    ma.merged = merged;
    ma.assign_out = assign_out;
    ma.inv_norm = reinterpret_cast<float *>(ws + p.off_inv_norm);
    ma.B = d->batch;
    ma.T = p.T;
    ma.D = d->feat_dim;
    ma.K = p.K;
    ma.is_bf16 = d->dtype == VSCAN_BF16;
    if (p.U > 0) VSCAN_LAUNCH("sim_argmax", launch_sim_argmax(ma, s));
    VSCAN_LAUNCH("merge", launch_merge(ma, s));
    return VSCAN_OK;
}

}  // namespace

// Pointer checks of the stage-2 tensors (host only).
static int check_llm_tensors(const vscan_llm_desc *d, const void *q, const void *k, const void *v,
                             const void *hidden, const int32_t *kept_idx, const void *k_out,
                             const void *v_out, const void *hidden_out, const float *scores_out) {
    if (!q || !k || !v || !hidden || (!kept_idx && d->keep > 0)) return VSCAN_ERR_NULL;
    const bool outs_null = !k_out && !v_out && !hidden_out;
    const bool outs_all = k_out && v_out && hidden_out;
    if (d->in_place ? !outs_null : !outs_all) return VSCAN_ERR_NULL;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(hidden) ||
        !aligned16(k_out) || !aligned16(v_out) || !aligned16(hidden_out))
        return VSCAN_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(kept_idx) & 3u) || (reinterpret_cast<uintptr_t>(scores_out) & 3u))
        return VSCAN_ERR_ALIGN;
    return VSCAN_OK;
}

namespace vscan {
// Everything vscan_llm_prune checks before it looks at its workspace, for the entry point that
// brings its own scratch.
int llm_prune_validate(const vscan_llm_desc *d, const void *q, const void *k, const void *v,
                       const void *hidden, const int32_t *kept_idx, const void *k_out,
                       const void *v_out, const void *hidden_out, const float *scores_out,
                       size_t *workspace_bytes) {
    LlmPlan p;
    const int rc = plan_llm(d, &p);
    if (rc != VSCAN_OK) return rc;
    *workspace_bytes = p.bytes;
    return check_llm_tensors(d, q, k, v, hidden, kept_idx, k_out, v_out, hidden_out, scores_out);
}
}  // namespace vscan

extern "C" {

int vscan_encoder_workspace_size(const vscan_encoder_desc *desc, int with_local_pair,
                                 size_t *bytes) {
    if (!bytes) return VSCAN_ERR_NULL;
    EncoderPlan p;
    const int rc = plan_encoder(desc, with_local_pair != 0, &p);
    if (rc != VSCAN_OK) return rc;
    *bytes = p.bytes;
    return VSCAN_OK;
}

static int encoder_reduce_impl(const vscan_encoder_desc *d, const void *q, const void *k,
                         const void *q_local, const void *k_local, const void *x,
                         int32_t *kept_idx, void *merged, int32_t *assign_out, float *scores_out,
                         void *workspace, size_t workspace_bytes, void *stream) {
    if ((q_local == nullptr) != (k_local == nullptr)) return VSCAN_ERR_NULL;
    const bool with_local = q_local != nullptr;
    EncoderPlan p;
    const int rc = plan_encoder(d, with_local, &p);
    if (rc != VSCAN_OK) return rc;
    if (!q || !k || !x || !kept_idx || !merged) return VSCAN_ERR_NULL;
    if (!aligned16(q) || !aligned16(k) || !aligned16(x) || !aligned16(merged) ||
        !aligned16(q_local) || !aligned16(k_local))
        return VSCAN_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(kept_idx) & 3u) || (reinterpret_cast<uintptr_t>(assign_out) & 3u) ||
        (reinterpret_cast<uintptr_t>(scores_out) & 3u))
        return VSCAN_ERR_ALIGN;
    if (!workspace || workspace_bytes < p.bytes) return VSCAN_ERR_WORKSPACE;
    if (!aligned16(workspace)) return VSCAN_ERR_ALIGN;
    if (d->batch == 0) return VSCAN_OK;

    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    unsigned char *ws = reinterpret_cast<unsigned char *>(workspace);
    const bool mean = d->score_mode == VSCAN_SCORE_MEAN_RECEIVED;

    ScoreArgs sa;
    sa.q = q;
    sa.k = k;
    sa.head_scores = reinterpret_cast<float *>(ws + p.off_head_global);
    sa.lse = reinterpret_cast<float *>(ws + p.off_lse);
    sa.BC = p.BC;
    sa.H = d->heads;
    sa.S = p.S;
    sa.dh = d->head_dim;
    sa.N = p.N;
    sa.has_cls = d->has_cls;
    sa.domain_all = d->softmax_domain == VSCAN_KEYS_ALL;
    sa.is_bf16 = d->dtype == VSCAN_BF16;
    sa.scale = resolve_scale(d->scale, d->head_dim);
    for (int pair = 0; pair < (with_local ? 2 : 1); ++pair) {
        if (pair == 1) {
            sa.q = q_local;
            sa.k = k_local;
            sa.head_scores = reinterpret_cast<float *>(ws + p.off_head_local);
        }
        if (mean) {
            VSCAN_LAUNCH("score_mean_lse", launch_score_mean_lse(sa, s));
            VSCAN_LAUNCH("score_mean_colsum", launch_score_mean_colsum(sa, s));
        } else {
            VSCAN_LAUNCH("score_cls", launch_score_cls(sa, s));
        }
    }

    return enqueue_encoder_tail(d, p, with_local, d->heads,
                                mean ? 1.0f / ((float)d->heads * (float)p.N) : 1.0f / (float)d->heads,
                                x, kept_idx, merged, assign_out, scores_out, ws, s);
}

int vscan_encoder_reduce(const vscan_encoder_desc *d, const void *q, const void *k,
                         const void *q_local, const void *k_local, const void *x,
                         int32_t *kept_idx, void *merged, int32_t *assign_out, float *scores_out,
                         void *workspace, size_t workspace_bytes, void *stream) {
    return finish("vscan_encoder_reduce", encoder_reduce_impl(d, q, k, q_local, k_local, x, kept_idx, merged, assign_out, scores_out, workspace, workspace_bytes, stream));
}

int vscan_encoder_fused_workspace_size(const vscan_encoder_desc *desc, int with_local_triple,
                                       size_t *bytes) {
    if (!bytes) return VSCAN_ERR_NULL;
    EncoderFusedPlan p;
    const int rc = plan_encoder_fused(desc, with_local_triple != 0, &p);
    if (rc != VSCAN_OK) return rc;
    *bytes = p.bytes;
    return VSCAN_OK;
}

static int encoder_reduce_fused_impl(const vscan_encoder_desc *d, const void *hidden, const void *w_q,
                               const void *w_k_t, const void *hidden_local,
                               const void *w_q_local, const void *w_k_t_local, const void *x,
                               int32_t *kept_idx, void *merged, int32_t *assign_out,
                               float *scores_out, void *workspace, size_t workspace_bytes,
                               void *stream) {
    const int n_local = (hidden_local != nullptr) + (w_q_local != nullptr) + (w_k_t_local != nullptr);
    if (n_local != 0 && n_local != 3) return VSCAN_ERR_NULL;
    const bool with_local = n_local == 3;
    EncoderFusedPlan p;
    const int rc = plan_encoder_fused(d, with_local, &p);
    if (rc != VSCAN_OK) return rc;
    if (!hidden || !w_q || !w_k_t || !x || !kept_idx || !merged) return VSCAN_ERR_NULL;
    if (!aligned16(hidden) || !aligned16(w_q) || !aligned16(w_k_t) || !aligned16(hidden_local) ||
        !aligned16(w_q_local) || !aligned16(w_k_t_local) || !aligned16(x) || !aligned16(merged))
        return VSCAN_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(kept_idx) & 3u) || (reinterpret_cast<uintptr_t>(assign_out) & 3u) ||
        (reinterpret_cast<uintptr_t>(scores_out) & 3u))
        return VSCAN_ERR_ALIGN;
    if (!workspace || workspace_bytes < p.bytes) return VSCAN_ERR_WORKSPACE;
    if (!aligned16(workspace)) return VSCAN_ERR_ALIGN;
    if (d->batch == 0) return VSCAN_OK;

    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    unsigned char *ws = reinterpret_cast<unsigned char *>(workspace);
    if (d->score_mode == VSCAN_SCORE_MEAN_RECEIVED) {
        // every token is a query: project Q and K of all tokens, then the two mean-attention
        // passes of the Q/K entry point on the fp32 result
        ScoreArgs sa;
        sa.q = ws + p.off_qf;
        sa.k = ws + p.off_kf;
        sa.lse = reinterpret_cast<float *>(ws + p.e.off_lse);
        sa.BC = p.e.BC;
        sa.H = d->heads;
        sa.S = p.e.S;
        sa.dh = d->head_dim;
        sa.N = p.e.N;
        sa.has_cls = d->has_cls;
        sa.domain_all = d->softmax_domain == VSCAN_KEYS_ALL;
        sa.is_bf16 = 0;
        sa.scale = resolve_scale(d->scale, d->head_dim);
        for (int pass = 0; pass < (with_local ? 2 : 1); ++pass) {
            ProjectArgs pa;
            pa.is_bf16 = d->dtype == VSCAN_BF16;
            pa.hidden = pass ? hidden_local : hidden;
            pa.BC = p.e.BC;
            pa.S = p.e.S;
            pa.Dh = d->feat_dim;
            pa.H = d->heads;
            pa.dh = d->head_dim;
            pa.w = pass ? w_q_local : w_q;
            pa.out = reinterpret_cast<float *>(ws + p.off_qf);
            VSCAN_LAUNCH("fused_project", launch_fused_project(pa, s));
            VSCAN_LAUNCH("fused_transpose", launch_transpose(pass ? w_k_t_local : w_k_t, ws + p.off_wk,
                                                            d->feat_dim, d->heads * d->head_dim,
                                                            elem_bytes(d->dtype), s));
            pa.w = ws + p.off_wk;
            pa.out = reinterpret_cast<float *>(ws + p.off_kf);
            VSCAN_LAUNCH("fused_project", launch_fused_project(pa, s));
            sa.head_scores = reinterpret_cast<float *>(ws + (pass ? p.e.off_head_local : p.e.off_head_global));
            VSCAN_LAUNCH("score_mean_lse", launch_score_mean_lse(sa, s));
            VSCAN_LAUNCH("score_mean_colsum", launch_score_mean_colsum(sa, s));
        }
        return enqueue_encoder_tail(d, p.e, with_local, d->heads,
                                    1.0f / ((float)d->heads * (float)p.e.N), x, kept_idx, merged,
                                    assign_out, scores_out, ws, s);
    }
    for (int pass = 0; pass < (with_local ? 2 : 1); ++pass) {
        FusedArgs fa;
        fa.is_bf16 = d->dtype == VSCAN_BF16;
        fa.hidden = pass ? hidden_local : hidden;
        fa.w_q = pass ? w_q_local : w_q;
        fa.w_k_t = pass ? w_k_t_local : w_k_t;
        fa.part = reinterpret_cast<float *>(ws + (pass ? p.e.off_head_local : p.e.off_head_global));
        fa.B = p.e.BC;
        fa.S = p.e.S;
        fa.Dh = d->feat_dim;
        fa.Hq = fa.Hkv = d->heads;
        fa.dh = d->head_dim;
        fa.Tq = 1;
        fa.q_row0 = 0;  // the [CLS] row
        fa.causal = 0;
        fa.vis_start = 1;
        fa.V = p.e.N;
        fa.k0 = p.k0;
        fa.nk = p.nk;
        fa.scale = resolve_scale(d->scale, d->head_dim);
        const int rc2 = enqueue_fused_scores(fa, p.f, ws, s);
        if (rc2 != VSCAN_OK) return rc2;
    }
    // the chain leaves one row of head sums per segment: [BC, 1, N]
    return enqueue_encoder_tail(d, p.e, with_local, 1, 1.0f / (float)d->heads, x, kept_idx, merged,
                                assign_out, scores_out, ws, s);
}

int vscan_encoder_reduce_fused(const vscan_encoder_desc *d, const void *hidden, const void *w_q,
                               const void *w_k_t, const void *hidden_local,
                               const void *w_q_local, const void *w_k_t_local, const void *x,
                               int32_t *kept_idx, void *merged, int32_t *assign_out,
                               float *scores_out, void *workspace, size_t workspace_bytes,
                               void *stream) {
    return finish("vscan_encoder_reduce_fused", encoder_reduce_fused_impl(d, hidden, w_q, w_k_t, hidden_local, w_q_local, w_k_t_local, x, kept_idx, merged, assign_out, scores_out, workspace, workspace_bytes, stream));
}

int vscan_llm_workspace_size(const vscan_llm_desc *desc, size_t *bytes) {
    if (!bytes) return VSCAN_ERR_NULL;
    LlmPlan p;
    const int rc = plan_llm(desc, &p);
    if (rc != VSCAN_OK) return rc;
    *bytes = p.bytes;
    return VSCAN_OK;
}

// Shared by the uniform and the ragged entry point.  `meta` (device) is NULL for a uniform
// batch; `max_out_rows` is the longest result, `out_rows` the row stride of the destinations.
static int run_llm(const vscan_llm_desc *d, const LlmPlan &p, const SeqMeta *meta, int max_out_rows,
                   int out_rows, const void *q, void *k, void *v, void *hidden, int32_t *kept_idx,
                   void *k_out, void *v_out, void *hidden_out, float *scores_out, void *workspace,
                   size_t workspace_bytes, void *stream) {
    const int rc_args = check_llm_tensors(d, q, k, v, hidden, kept_idx, k_out, v_out, hidden_out,
                                          scores_out);
    if (rc_args != VSCAN_OK) return rc_args;
    if (!workspace || workspace_bytes < p.bytes) return VSCAN_ERR_WORKSPACE;
    if (!aligned16(workspace)) return VSCAN_ERR_ALIGN;
    if (d->batch == 0) return VSCAN_OK;

    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    unsigned char *ws = reinterpret_cast<unsigned char *>(workspace);

    LlmScoreArgs sa;
    sa.q = q;
    sa.k = k;
    sa.part = reinterpret_cast<float *>(ws + p.off_part);
    sa.B = d->batch;
    sa.Hq = d->q_heads;
    sa.Hkv = d->kv_heads;
    sa.Tq = d->n_query;
    sa.S = d->seq_len;
    sa.dh = d->head_dim;
    sa.vis_start = d->vis_start;
    sa.V = d->vis_len;
    sa.domain_all = d->softmax_domain == VSCAN_KEYS_ALL;
    sa.is_bf16 = d->dtype == VSCAN_BF16;
    sa.scale = resolve_scale(d->scale, d->head_dim);
    sa.meta = meta;
    sa.split_e = reinterpret_cast<float *>(ws + p.off_split_e);
    sa.split_stats = reinterpret_cast<float *>(ws + p.off_split_stats);
    VSCAN_LAUNCH("llm_score", launch_llm_score(sa, s));

    LlmSelectArgs se;
    se.part = sa.part;
    se.B = d->batch;
    se.Hkv = d->kv_heads;
    se.V = d->vis_len;
    se.keep = d->keep;
    se.norm = 1.0f / ((float)d->n_query * (float)d->q_heads);
    se.kept_idx = kept_idx;
    se.scores_out = scores_out;
    se.meta = meta;
    VSCAN_LAUNCH("llm_select", launch_llm_select(se, s));

    CompactArgs ca;
    ca.k = k;
    ca.v = v;
    ca.hidden = hidden;
    ca.k_out = k_out;
    ca.v_out = v_out;
    ca.hidden_out = hidden_out;
    // The compaction kernels fetch an index for every row from a clamped position, so the
    // table must be readable even when nothing is kept: the (never used) value then comes
    // from the start of the workspace.
    ca.kept_idx = d->keep > 0 ? kept_idx : reinterpret_cast<const int32_t *>(ws + p.off_part);
    ca.B = d->batch;
    ca.Hkv = d->kv_heads;
    ca.S = d->seq_len;
    ca.dh = d->head_dim;
    ca.Dh = d->hidden;
    ca.vis_start = d->vis_start;
    ca.V = d->vis_len;
    ca.keep = d->keep;
    ca.elem_bytes = elem_bytes(d->dtype);
    ca.in_place = d->in_place;
    ca.out_rows = out_rows;
    ca.max_out_rows = max_out_rows;
    ca.meta = meta;
    VSCAN_LAUNCH("compact", launch_compact(ca, s));
    return VSCAN_OK;
}

static int llm_prune_impl(const vscan_llm_desc *d, const void *q, void *k, void *v, void *hidden,
                    int32_t *kept_idx, void *k_out, void *v_out, void *hidden_out,
                    float *scores_out, void *workspace, size_t workspace_bytes, void *stream) {
    LlmPlan p;
    const int rc = plan_llm(d, &p);
    if (rc != VSCAN_OK) return rc;
    return run_llm(d, p, nullptr, p.S_out, d->in_place ? d->seq_len : p.S_out, q, k, v, hidden,
                   kept_idx, k_out, v_out, hidden_out, scores_out, workspace, workspace_bytes,
                   stream);
}

int vscan_llm_prune(const vscan_llm_desc *d, const void *q, void *k, void *v, void *hidden,
                    int32_t *kept_idx, void *k_out, void *v_out, void *hidden_out,
                    float *scores_out, void *workspace, size_t workspace_bytes, void *stream) {
    return finish("vscan_llm_prune", llm_prune_impl(d, q, k, v, hidden, kept_idx, k_out, v_out, hidden_out, scores_out, workspace, workspace_bytes, stream));
}

static int check_seq_meta(const vscan_llm_desc *d, const vscan_seq_meta *meta_host,
                          const vscan_seq_meta *meta_device, int *max_out_rows);

static int llm_prune_ragged_impl(const vscan_llm_desc *d, const vscan_seq_meta *meta_host,
                           const vscan_seq_meta *meta_device, const void *q, void *k, void *v,
                           void *hidden, int32_t *kept_idx, void *k_out, void *v_out,
                           void *hidden_out, float *scores_out, void *workspace,
                           size_t workspace_bytes, void *stream) {
    if (!d) return VSCAN_ERR_NULL;
    if (d->struct_size != sizeof(vscan_llm_desc)) return VSCAN_ERR_VERSION;
    // the descriptor's lengths are capacities here; its vis_start has no meaning
    vscan_llm_desc caps = *d;
    caps.vis_start = 0;
    LlmPlan p;
    const int rc = plan_llm(&caps, &p);
    if (rc != VSCAN_OK) return rc;
    int max_out_rows = 0;
    const int rc2 = check_seq_meta(d, meta_host, meta_device, &max_out_rows);
    if (rc2 != VSCAN_OK) return rc2;
    static_assert(sizeof(SeqMeta) == sizeof(vscan_seq_meta), "same layout");
    return run_llm(&caps, p, reinterpret_cast<const SeqMeta *>(meta_device), max_out_rows,
                   d->seq_len, q, k, v, hidden, kept_idx, k_out, v_out, hidden_out, scores_out,
                   workspace, workspace_bytes, stream);
}

int vscan_llm_prune_ragged(const vscan_llm_desc *d, const vscan_seq_meta *meta_host,
                           const vscan_seq_meta *meta_device, const void *q, void *k, void *v,
                           void *hidden, int32_t *kept_idx, void *k_out, void *v_out,
                           void *hidden_out, float *scores_out, void *workspace,
                           size_t workspace_bytes, void *stream) {
    return finish("vscan_llm_prune_ragged", llm_prune_ragged_impl(d, meta_host, meta_device, q, k, v, hidden, kept_idx, k_out, v_out, hidden_out, scores_out, workspace, workspace_bytes, stream));
}

int vscan_llm_fused_workspace_size(const vscan_llm_desc *desc, size_t *bytes) {
    if (!bytes) return VSCAN_ERR_NULL;
    FusedPlan p;
    const int rc = plan_fused(desc, &p);
    if (rc != VSCAN_OK) return rc;
    *bytes = p.bytes;
    return VSCAN_OK;
}

// Shared by the uniform and the ragged form.  `meta` (device) is NULL for a uniform batch;
// `max_out_rows` is the longest result, `out_rows` the row stride of hidden_out.
static int run_llm_fused(const vscan_llm_desc *d, const FusedPlan &p, const SeqMeta *meta,
                         int max_out_rows, int out_rows, void *hidden, const void *w_q,
                         const void *w_k_t, int32_t *kept_idx, void *hidden_out, float *scores_out,
                         void *workspace, size_t workspace_bytes, void *stream) {
    if (!hidden || !w_q || !w_k_t || (!kept_idx && d->keep > 0)) return VSCAN_ERR_NULL;
    if (d->in_place ? hidden_out != nullptr : hidden_out == nullptr) return VSCAN_ERR_NULL;
    if (!aligned16(hidden) || !aligned16(w_q) || !aligned16(w_k_t) || !aligned16(hidden_out))
        return VSCAN_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(kept_idx) & 3u) || (reinterpret_cast<uintptr_t>(scores_out) & 3u))
        return VSCAN_ERR_ALIGN;
    if (!workspace || workspace_bytes < p.bytes) return VSCAN_ERR_WORKSPACE;
    if (!aligned16(workspace)) return VSCAN_ERR_ALIGN;
    if (d->batch == 0) return VSCAN_OK;

    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    unsigned char *ws = reinterpret_cast<unsigned char *>(workspace);

    FusedArgs fa;
    fa.is_bf16 = d->dtype == VSCAN_BF16;
    fa.hidden = hidden;
    fa.w_q = w_q;
    fa.w_k_t = w_k_t;
    fa.part = reinterpret_cast<float *>(ws + p.off_part);
    fa.B = d->batch;
    fa.S = d->seq_len;
    fa.Dh = d->hidden;
    fa.Hq = d->q_heads;
    fa.Hkv = d->kv_heads;
    fa.dh = d->head_dim;
    fa.Tq = d->n_query;
    fa.q_row0 = d->seq_len - d->n_query;  // the last positions
    // over all keys each query attends causally: up to and including its own position
    fa.causal = d->softmax_domain == VSCAN_KEYS_ALL;
    fa.vis_start = d->vis_start;
    fa.V = d->vis_len;
    fa.k0 = p.k0;
    fa.nk = p.nk;
    fa.scale = resolve_scale(d->scale, d->head_dim);
    fa.meta = meta;
    const int rc2 = enqueue_fused_scores(fa, p.f, ws, s);
    if (rc2 != VSCAN_OK) return rc2;

    LlmSelectArgs se;
    se.part = fa.part;
    se.B = d->batch;
    se.Hkv = 1;
    se.V = d->vis_len;
    se.keep = d->keep;
    se.norm = 1.0f / (float)p.R;
    se.kept_idx = kept_idx;
    se.scores_out = scores_out;
    se.meta = meta;
    VSCAN_LAUNCH("llm_select", launch_llm_select(se, s));

    CompactArgs ca;
    ca.k = ca.v = ca.k_out = ca.v_out = nullptr;
    ca.hidden = hidden;
    ca.hidden_out = hidden_out;
    ca.kept_idx = d->keep > 0 ? kept_idx : reinterpret_cast<const int32_t *>(ws + p.off_part);
    ca.B = d->batch;
    ca.Hkv = 0;  // no K / V strips
    ca.S = d->seq_len;
    ca.dh = d->head_dim;
    ca.Dh = d->hidden;
    ca.vis_start = d->vis_start;
    ca.V = d->vis_len;
    ca.keep = d->keep;
    ca.elem_bytes = elem_bytes(d->dtype);
    ca.in_place = d->in_place;
    ca.out_rows = out_rows;
    ca.max_out_rows = max_out_rows;
    ca.meta = meta;
    VSCAN_LAUNCH("compact", launch_compact(ca, s));
    return VSCAN_OK;
}

static int llm_prune_fused_impl(const vscan_llm_desc *d, void *hidden, const void *w_q,
                          const void *w_k_t, int32_t *kept_idx, void *hidden_out,
                          float *scores_out, void *workspace, size_t workspace_bytes,
                          void *stream) {
    FusedPlan p;
    const int rc = plan_fused(d, &p);
    if (rc != VSCAN_OK) return rc;
    return run_llm_fused(d, p, nullptr, p.S_out, d->in_place ? d->seq_len : p.S_out, hidden, w_q,
                         w_k_t, kept_idx, hidden_out, scores_out, workspace, workspace_bytes,
                         stream);
}

int vscan_llm_prune_fused(const vscan_llm_desc *d, void *hidden, const void *w_q,
                          const void *w_k_t, int32_t *kept_idx, void *hidden_out,
                          float *scores_out, void *workspace, size_t workspace_bytes,
                          void *stream) {
    return finish("vscan_llm_prune_fused", llm_prune_fused_impl(d, hidden, w_q, w_k_t, kept_idx, hidden_out, scores_out, workspace, workspace_bytes, stream));
}

// Validation of a ragged batch's host table against the capacities; *max_out_rows receives the
// longest result.
static int check_seq_meta(const vscan_llm_desc *d, const vscan_seq_meta *meta_host,
                          const vscan_seq_meta *meta_device, int *max_out_rows) {
    if (d->batch > 0 && (!meta_host || !meta_device)) return VSCAN_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(meta_device) & 3u) return VSCAN_ERR_ALIGN;
    *max_out_rows = 0;
    for (int b = 0; b < d->batch; ++b) {
        const vscan_seq_meta &m = meta_host[b];
        if (m.seq_len < 1 || m.seq_len > d->seq_len || m.vis_start < 0 || m.vis_len < 1 ||
            m.vis_len > d->vis_len)
            return VSCAN_ERR_SHAPE;
        if ((int64_t)m.vis_start + m.vis_len + d->n_query > m.seq_len) return VSCAN_ERR_SHAPE;
        if (m.keep < 0 || m.keep > m.vis_len || m.keep > d->keep) return VSCAN_ERR_BUDGET;
        *max_out_rows = std::max(*max_out_rows, m.seq_len - m.vis_len + m.keep);
    }
    return VSCAN_OK;
}

static int llm_prune_fused_ragged_impl(const vscan_llm_desc *d, const vscan_seq_meta *meta_host,
                                 const vscan_seq_meta *meta_device, void *hidden, const void *w_q,
                                 const void *w_k_t, int32_t *kept_idx, void *hidden_out,
                                 float *scores_out, void *workspace, size_t workspace_bytes,
                                 void *stream) {
    if (!d) return VSCAN_ERR_NULL;
    if (d->struct_size != sizeof(vscan_llm_desc)) return VSCAN_ERR_VERSION;
    vscan_llm_desc caps = *d;  // lengths are capacities; vis_start has no meaning
    caps.vis_start = 0;
    FusedPlan p;
    const int rc = plan_fused(&caps, &p);
    if (rc != VSCAN_OK) return rc;
    int max_out_rows = 0;
    const int rc2 = check_seq_meta(d, meta_host, meta_device, &max_out_rows);
    if (rc2 != VSCAN_OK) return rc2;
    return run_llm_fused(&caps, p, reinterpret_cast<const SeqMeta *>(meta_device), max_out_rows,
                         d->seq_len, hidden, w_q, w_k_t, kept_idx, hidden_out, scores_out,
                         workspace, workspace_bytes, stream);
}

int vscan_llm_prune_fused_ragged(const vscan_llm_desc *d, const vscan_seq_meta *meta_host,
                                 const vscan_seq_meta *meta_device, void *hidden, const void *w_q,
                                 const void *w_k_t, int32_t *kept_idx, void *hidden_out,
                                 float *scores_out, void *workspace, size_t workspace_bytes,
                                 void *stream) {
    return finish("vscan_llm_prune_fused_ragged", llm_prune_fused_ragged_impl(d, meta_host, meta_device, hidden, w_q, w_k_t, kept_idx, hidden_out, scores_out, workspace, workspace_bytes, stream));
}

int vscan_profile_enable(int on) {
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    g_prof_on.store(on != 0, std::memory_order_relaxed);
    return VSCAN_OK;
}

int vscan_profile_read(vscan_kernel_time *out, int capacity, int *count) {
    if (!out || !count || capacity < 0) return VSCAN_ERR_NULL;
    std::vector<ProfRecord> recs;
    {
        std::lock_guard<std::mutex> lock(g_prof_mutex);
        recs.swap(g_prof_records);
    }
    int n = 0, rc = VSCAN_OK;
    for (const ProfRecord &r : recs) {
        float ms = 0.f;
        if (hipEventSynchronize(r.stop) != hipSuccess ||
            hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess)
            rc = VSCAN_ERR_HIP;
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
        int i = 0;
        while (i < n && strcmp(out[i].name, r.name) != 0) ++i;
        if (i == n) {
            if (n == capacity) continue;
            memset(&out[n], 0, sizeof(out[n]));
            strncpy(out[n].name, r.name, sizeof(out[n].name) - 1);
            ++n;
        }
        out[i].launches += 1;
        out[i].total_ms += ms;
    }
    *count = n;
    return rc;
}

const char *vscan_status_string(int status) {
    switch (status) {
        case VSCAN_OK: return "ok";
        case VSCAN_ERR_NULL: return "a required pointer is NULL (or an optional pair is half given)";
        case VSCAN_ERR_SHAPE: return "a dimension is out of range or inconsistent";
        case VSCAN_ERR_BUDGET: return "a keep budget does not fit the tokens or windows";
        case VSCAN_ERR_DTYPE: return "unknown dtype, score mode or softmax domain";
        case VSCAN_ERR_ALIGN: return "a tensor pointer is not sufficiently aligned";
        case VSCAN_ERR_WORKSPACE: return "workspace is missing or too small";
        case VSCAN_ERR_HIP: return "a HIP runtime call failed";
        case VSCAN_ERR_VERSION: return "descriptor struct_size does not match this library";
        case VSCAN_ERR_UNSUPPORTED: return "valid request outside the limits of the kernels";
        default: return "unknown status";
    }
}

uint32_t vscan_version(void) { return VSCAN_VERSION; }

}  // extern "C"
