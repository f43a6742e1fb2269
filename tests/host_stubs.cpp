// Stand-ins for the kernel launchers, for a CPU-only build of the host layer (api.cpp,
// budget.cpp) under AddressSanitizer and UndefinedBehaviorSanitizer.  Nothing here launches or
// dereferences anything.  Each stand-in checks what the host layer hands to a launcher: every
// scratch region (start and extent, worked out from the dimensions in the argument struct) must
// lie inside the workspace window the test announced, 16-byte aligned, and the regions of one
// call must not overlap.  The test reads the tally through vscan_test_report.
#include <stdint.h>
#include <stdio.h>

#include <algorithm>
#include <utility>
#include <vector>

#include "../paper_2505_22654_amd/csrc/fused.hpp"
#include "../paper_2505_22654_amd/csrc/launch.hpp"

namespace {
uintptr_t g_lo = 0, g_hi = 0;
int g_calls = 0, g_regions = 0, g_violations = 0;

void region(const char *who, const char *what, const void *p, size_t bytes) {
    ++g_regions;
    const uintptr_t a = reinterpret_cast<uintptr_t>(p);
    if (!p || (a & 15u) || a < g_lo || a + bytes > g_hi || a + bytes < a) {
        ++g_violations;
        fprintf(stderr, "host_stubs: %s: %s [%p, +%zu) outside the window or unaligned\n", who, what,
                p, bytes);
    }
}
// regions that must be distinct from one another within a call
void distinct(const char *who, std::vector<std::pair<const void *, size_t>> rs) {
    std::vector<std::pair<uintptr_t, uintptr_t>> v;
    for (auto &r : rs)
        if (r.first && r.second) v.push_back({(uintptr_t)r.first, (uintptr_t)r.first + r.second});
    std::sort(v.begin(), v.end());
    for (size_t i = 1; i < v.size(); ++i)
        if (v[i].first < v[i - 1].second) {
            ++g_violations;
            fprintf(stderr, "host_stubs: %s: scratch regions overlap\n", who);
        }
}
}  // namespace

extern "C" void vscan_test_window(const void *lo, size_t bytes) {
    g_lo = reinterpret_cast<uintptr_t>(lo);
    g_hi = g_lo + bytes;
}
extern "C" void vscan_test_report(int *calls, int *regions, int *violations) {
    *calls = g_calls;
    *regions = g_regions;
    *violations = g_violations;
}

namespace vscan {

static void check_score(const char *who, const ScoreArgs &a, bool mean) {
    ++g_calls;
    const size_t n = (size_t)a.BC * a.H * a.N * sizeof(float);
    region(who, "head_scores", a.head_scores, n);
    if (mean) {
        region(who, "lse", a.lse, n);
        distinct(who, {{a.head_scores, n}, {a.lse, n}});
    }
}
hipError_t launch_score_cls(const ScoreArgs &a, hipStream_t) {
    check_score("score_cls", a, false);
    return hipSuccess;
}
hipError_t launch_score_mean_lse(const ScoreArgs &a, hipStream_t) {
    check_score("score_mean_lse", a, true);
    return hipSuccess;
}
hipError_t launch_score_mean_colsum(const ScoreArgs &a, hipStream_t) {
    check_score("score_mean_colsum", a, true);
    return hipSuccess;
}

hipError_t launch_encoder_select(const EncSelectArgs &a, hipStream_t) {
    ++g_calls;
    const size_t N = (size_t)a.gh * a.gw, BC = (size_t)a.B * a.C;
    const size_t K = (size_t)a.C * ((size_t)a.wr * a.wc * a.kw + a.kg);
    const size_t head = BC * a.H * N * sizeof(float);
    region("encoder_select", "head_global", a.head_global, head);
    if (a.head_local) region("encoder_select", "head_local", a.head_local, head);
    region("encoder_select", "drop_idx", a.drop_idx, (size_t)a.B * (a.C * N - K) * 4);
    region("encoder_select", "best", a.best, BC * N * 8);
    region("encoder_select", "pre_key", a.pre_key_ws, BC * N * 4);
    region("encoder_select", "pre_flag", a.pre_flag_ws, BC * N);
    distinct("encoder_select", {{a.head_global, head},
                                {a.head_local, head},
                                {a.drop_idx, (size_t)a.B * (a.C * N - K) * 4},
                                {a.best, BC * N * 8},
                                {a.pre_key_ws, BC * N * 4},
                                {a.pre_flag_ws, BC * N}});
    return hipSuccess;
}
size_t encoder_select_lds_bytes(int N, int has_local) {
    return 1024 + (size_t)N * 4 * (has_local ? 2 : 1) + (size_t)N;
}

static void check_merge(const char *who, const MergeArgs &a) {
    ++g_calls;
    const size_t U = (size_t)a.T - a.K;
    region(who, "drop_idx", a.drop_idx, (size_t)a.B * U * 4);
    region(who, "best", a.best, (size_t)a.B * a.T * 8);
    region(who, "inv_norm", a.inv_norm, (size_t)a.B * a.K * 4);
    distinct(who, {{a.drop_idx, (size_t)a.B * U * 4},
                   {a.best, (size_t)a.B * a.T * 8},
                   {a.inv_norm, (size_t)a.B * a.K * 4}});
}
hipError_t launch_sim_argmax(const MergeArgs &a, hipStream_t) {
    check_merge("sim_argmax", a);
    return hipSuccess;
}
hipError_t launch_merge(const MergeArgs &a, hipStream_t) {
    check_merge("merge", a);
    return hipSuccess;
}

int llm_score_split_chunks(int B, int Hkv, int rows, int nk, bool ragged) {
    if (ragged || rows > 16 || nk < 1024 || (int64_t)B * Hkv > 64) return 0;
    return (nk + 63) / 64;
}
bool llm_score_supported(int rows, int, int row_bytes) { return rows <= 64 && row_bytes <= 512; }
hipError_t launch_llm_score(const LlmScoreArgs &a, hipStream_t) {
    ++g_calls;
    const size_t items = (size_t)a.B * a.Hkv, rows = (size_t)(a.Hq / a.Hkv) * a.Tq;
    const size_t part = items * a.V * 4;
    region("llm_score", "part", a.part, part);
    const int nk = a.domain_all ? a.S : a.V;
    const int chunks = llm_score_split_chunks(a.B, a.Hkv, (int)rows, nk, a.meta != nullptr);
    if (chunks > 0) {
        const size_t e = items * rows * a.V * 4, st = items * chunks * rows * 2 * 4;
        region("llm_score", "split_e", a.split_e, e);
        region("llm_score", "split_stats", a.split_stats, st);
        distinct("llm_score", {{a.part, part}, {a.split_e, e}, {a.split_stats, st}});
    }
    return hipSuccess;
}
hipError_t launch_llm_select(const LlmSelectArgs &a, hipStream_t) {
    ++g_calls;
    region("llm_select", "part", a.part, (size_t)a.B * a.Hkv * a.V * 4);
    return hipSuccess;
}
size_t llm_select_lds_bytes(int V) { return 1024 + (size_t)V * 5; }
hipError_t launch_compact(const CompactArgs &, hipStream_t) {
    ++g_calls;
    return hipSuccess;
}

int fused_ksplit(int, int, int, int k_elems, int) { return k_elems >= 512 ? 2 : 1; }
static hipError_t check_fused(const char *who, const FusedArgs &a) {
    ++g_calls;
    const size_t M = (size_t)a.B * a.Tq, N = (size_t)a.Hq * a.dh, R = (size_t)a.Hq * a.Tq;
    const size_t cq = (size_t)a.ks_q * M * N * 4, qp = a.is_bf16 ? 3 * M * N * 2 : M * N * 4;
    const size_t qt = (a.is_bf16 ? (size_t)kFusedQtPlanes * 2 : 4) * a.B * R * a.Dh;
    const size_t cl = (size_t)a.ks_l * a.B * R * a.nk * 4;
    region(who, "c_q", a.c_q, cq);
    region(who, "q_planes", a.q_planes, qp);
    region(who, "qt_planes", a.qt_planes, qt);
    region(who, "c_l", a.c_l, cl);
    region(who, "part", a.part, (size_t)a.B * a.V * 4);
    distinct(who, {{a.c_q, cq}, {a.q_planes, qp}, {a.qt_planes, qt}, {a.c_l, cl},
                   {a.part, (size_t)a.B * a.V * 4}});
    return hipSuccess;
}
hipError_t launch_fused_project(const ProjectArgs &a, hipStream_t) {
    ++g_calls;
    region("fused_project", "out", a.out, (size_t)a.BC * a.H * a.S * a.dh * 4);
    return hipSuccess;
}
hipError_t launch_transpose(const void *, void *out, int rows, int cols, int es, hipStream_t) {
    ++g_calls;
    region("fused_transpose", "out", out, (size_t)rows * cols * es);
    return hipSuccess;
}
hipError_t launch_fused_q(const FusedArgs &a, hipStream_t) { return check_fused("fused_q", a); }
hipError_t launch_fused_split_q(const FusedArgs &a, hipStream_t) { return check_fused("fused_split_q", a); }
hipError_t launch_fused_qt(const FusedArgs &a, hipStream_t) { return check_fused("fused_qt", a); }
hipError_t launch_fused_logits(const FusedArgs &a, hipStream_t) { return check_fused("fused_logits", a); }
hipError_t launch_fused_softmax(const FusedArgs &a, hipStream_t) { return check_fused("fused_softmax", a); }
hipError_t launch_fused_colsum(const FusedArgs &a, hipStream_t) { return check_fused("fused_colsum", a); }

}  // namespace vscan
