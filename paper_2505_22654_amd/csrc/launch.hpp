// Host-side launch interface between the C ABI layer and the kernel files.
// Every launcher enqueues on the given stream and returns hipGetLastError().
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

namespace vscan {

// Dynamic LDS above 64 KB has to be allowed per kernel.  The limit is raised to the most one
// workgroup can have, once per kernel instantiation and device: `done` is a static of the
// calling instantiation, one bit per device.  Later launches only read the bit.  A kernel that
// also has static LDS passes a `limit` that leaves room for it.
constexpr int kMaxDynamicLds = 160 * 1024;
template <typename Kernel>
inline hipError_t allow_large_lds(Kernel kernel, std::atomic<uint64_t> &done,
                                  int limit = kMaxDynamicLds) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, limit);
    if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
    return e;
}


// encoder attention scoring (Eq. 1-2)
struct ScoreArgs {
    const void *q, *k;    // [BC, H, S, dh]
    float *head_scores;   // [BC, H, N] un-averaged per-head scores
    float *lse;           // [BC, H, N] scratch, mean mode only
    int BC, H, S, dh, N;
    int has_cls, domain_all, is_bf16;
    float scale;
};
hipError_t launch_score_cls(const ScoreArgs &a, hipStream_t s);
hipError_t launch_score_mean_lse(const ScoreArgs &a, hipStream_t s);     // pass 1
hipError_t launch_score_mean_colsum(const ScoreArgs &a, hipStream_t s);  // pass 2

// local + global selection (Eq. 2-3, footnote on priority)
struct EncSelectArgs {
    const float *head_global;  // [BC, H, N]
    const float *head_local;   // [BC, H, N] or NULL (= head_global)
    int B, C, H, gh, gw, wr, wc;
    int kw;                    // per window
    int kg;                    // per segment, remainder of the local budget included
    float norm;                // 1/H or 1/(H*N)
    int32_t *kept_idx;         // [B, C*(W*kw+kg)]
    int32_t *drop_idx;         // [B, C*N - K]
    uint64_t *best;            // [B, C*N] packed (similarity key, ~slot)
    float *scores_out;         // optional [B, C*N]
    // scratch for large segments, where the local scan runs as a kernel of its own:
    // global-scan keys [BC, N] and local-scan flags [BC, N]
    uint32_t *pre_key_ws = nullptr;
    uint8_t *pre_flag_ws = nullptr;
    // set by the launcher for the second kernel of that form
    const uint32_t *pre_key = nullptr;
    const uint8_t *pre_flag = nullptr;
};
hipError_t launch_encoder_select(const EncSelectArgs &a, hipStream_t s);
size_t encoder_select_lds_bytes(int N, int has_local);

// cosine assignment (Sec. 4.1 "Token Merging") and Eq. 4
struct MergeArgs {
    const void *x;             // [B, T, D]
    const int32_t *kept_idx;   // [B, K]
    const int32_t *drop_idx;   // [B, U]
    uint64_t *best;            // [B, T]
    void *merged;              // [B, K, D]
    int32_t *assign_out;       // optional [B, T]
    float *inv_norm;           // [B, K] scratch: 1 / ||x_s|| of the kept rows (large form only)
    int B, T, D, K, is_bf16;
};
hipError_t launch_sim_argmax(const MergeArgs &a, hipStream_t s);
hipError_t launch_merge(const MergeArgs &a, hipStream_t s);

// Per-sequence lengths of a ragged stage-2 batch (same layout as vscan_seq_meta).  Where an
// args struct carries a non-NULL `meta` (a DEVICE array of B entries), the kernels take
// seq_len / vis_start / vis_len / keep of sequence b from meta[b]; the struct's own S, V, keep
// then are capacities: tensor strides and LDS sizes.
struct SeqMeta {
    int32_t seq_len, vis_start, vis_len, keep;
};

// stage 2 scoring (Eq. 5)
struct LlmScoreArgs {
    const void *q;             // [B, Hq, Tq, dh]
    const void *k;             // [B, Hkv, S, dh]
    float *part;               // [B, Hkv, V] un-averaged sums over the query rows of a kv head
    int B, Hq, Hkv, Tq, S, dh, vis_start, V;
    int domain_all, is_bf16;
    float scale;
    const SeqMeta *meta = nullptr;
    // scratch of the form that cuts long key domains into chunks (llm_score_split_chunks > 0):
    // e [B*Hkv, rows, V] and per-chunk (maximum, sum) pairs [B*Hkv, chunks, rows, 2]
    float *split_e = nullptr, *split_stats = nullptr;
};
hipError_t launch_llm_score(const LlmScoreArgs &a, hipStream_t s);
int llm_score_split_chunks(int B, int Hkv, int rows, int nk, bool ragged);
// rows = (Hq/Hkv)*Tq query rows per kv head, nk = keys in the softmax domain
bool llm_score_supported(int rows, int nk, int row_bytes);

struct LlmSelectArgs {
    const float *part;         // [B, Hkv, V]
    int B, Hkv, V, keep;
    float norm;                // 1/(Tq*Hq)
    int32_t *kept_idx;         // [B, keep]; ragged: entries past a sequence's own keep are -1
    float *scores_out;         // optional [B, V]
    const SeqMeta *meta = nullptr;
};
hipError_t launch_llm_select(const LlmSelectArgs &a, hipStream_t s);
size_t llm_select_lds_bytes(int V);

// order-preserving compaction ("Remarks on KV Cache")
struct CompactArgs {
    void *k, *v, *hidden;              // sources (and destinations when in_place)
    void *k_out, *v_out, *hidden_out;  // NULL when in_place
    const int32_t *kept_idx;           // [B, keep]; at least one readable int when keep == 0
    int B, Hkv, S, dh, Dh, vis_start, V, keep, elem_bytes, in_place;
    // rows between consecutive slabs of the destinations: S - V + keep for the dense
    // out-of-place result, S when compacting in place or into tensors shaped like the inputs
    int out_rows;
    int max_out_rows;  // rows of the longest result (S - V + keep when every sequence is alike)
    const SeqMeta *meta = nullptr;
};
hipError_t launch_compact(const CompactArgs &a, hipStream_t s);

}  // namespace vscan
