// Attention scoring of encoder tokens (Sec. 4.1 "Global Scan", Eq. 1-2).
//
// Both modes write one UN-AVERAGED value per (segment, head, patch token) into
// `head_scores` [BC, H, N]; the selection kernel sums the heads in a fixed order
// and applies the 1/H (or 1/(H*N)) factor of Eq. 2.
//
//   [CLS] mode   head_scores[h][j] = softmax_j(scale * q_CLS^h . k_j^h)
//   mean mode    head_scores[h][j] = sum_i softmax_row_i(scale * q_i^h . k^h)_j
//                (two passes over Q K^T on the matrix cores: row log-sum-exp,
//                then column sums of exp(s - lse_i); the N x N matrix is never
//                stored)
#include "common.hpp"
#include "launch.hpp"

namespace vscan {

// ---------------------------------------------------------------------------
// [CLS] row.  One workgroup per (segment, head): a batched GEMV over the keys,
// bound by reading K once.  A key row is split into 16-byte pieces over adjacent
// lanes, so a wave reads whole rows contiguously.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void score_cls_generic_kernel(const T *__restrict__ q,
                                                        const T *__restrict__ k,
                                                        float *__restrict__ head_scores, int H,
                                                        int S, int dh, int first_key, int col0,
                                                        int N, float scale_log2e) {
    constexpr int E = ElemTraits<T>::kPer16B;
    extern __shared__ __align__(16) unsigned char smem[];
    float *red = reinterpret_cast<float *>(smem);  // 16 floats
    float *qf = red + 16;                           // dh floats (dh <= 256)
    float *z = qf + 256;                            // n_keys floats

    const int h = blockIdx.x, bc = blockIdx.y;
    const int64_t head_row0 = ((int64_t)bc * H + h) * S;
    const T *qrow = q + head_row0 * dh;
    const T *kbase = k + (head_row0 + first_key) * dh;
    const int n_keys = S - first_key;
    const int tid = threadIdx.x;

    for (int e = tid; e < dh; e += blockDim.x) qf[e] = load_elem<T>(qrow + e) * scale_log2e;
    __syncthreads();

    const int cpr = dh / E;          // 16-byte pieces per key row (<= 64)
    const int rpw = kWave / cpr;     // key rows per wave per step
    const int lane = lane_id();
    const int row_in_wave = lane / cpr;
    const int piece = lane - row_in_wave * cpr;
    const bool active = row_in_wave < rpw;
    const int seg0 = row_in_wave * cpr;
    float qreg[E];
#pragma unroll
    for (int e = 0; e < E; ++e) qreg[e] = active ? qf[piece * E + e] : 0.f;

    const int nw = blockDim.x / kWave;
    constexpr int UNR = 4;
    const int64_t row_bytes = (int64_t)dh * sizeof(T);
    for (int base = wave_id() * rpw; base < n_keys; base += nw * rpw * UNR) {
        uint4 raw[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int row = base + u * nw * rpw + row_in_wave;
            raw[u] = load16_stream_guard(kbase, row * row_bytes + piece * 16, active && row < n_keys);
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int row = base + u * nw * rpw + row_in_wave;
            float kv[E];
            unpack16<T>(raw[u], kv);
            float part = 0.f;
#pragma unroll
            for (int e = 0; e < E; ++e) part = fmaf(kv[e], qreg[e], part);
            float tot = 0.f;
            for (int d = 0; d < cpr; ++d) tot += __shfl(part, (seg0 + d) & (kWave - 1), kWave);
            if (active && piece == 0 && row < n_keys) z[row] = tot;
        }
    }
    __syncthreads();

    float m = -INFINITY;
    for (int j = tid; j < n_keys; j += blockDim.x) m = fmaxf(m, z[j]);
    m = block_max(m, red);
    float sum = 0.f;
    for (int j = tid; j < n_keys; j += blockDim.x) {
        const float e = __builtin_amdgcn_exp2f(z[j] - m);
        z[j] = e;
        sum += e;
    }
    sum = block_sum(sum, red);
    const float inv = 1.0f / sum;
    float *out = head_scores + ((int64_t)bc * H + h) * N;
    for (int j = tid; j < N; j += blockDim.x) out[j] = z[col0 + j] * inv;
}

// Same computation for rows whose piece count is a power of two (every common head
// size).  The key block is read as one flat, fully coalesced stream with up to 16
// independent 16-byte loads per thread in flight: at these sizes the kernel's time
// is the number of serialised memory round-trips, so all of them are issued at once.
template <typename T, int LOG2_CPR, int UNR>
__global__ __launch_bounds__(256) void score_cls_kernel(const T *__restrict__ q,
                                                        const T *__restrict__ k,
                                                        float *__restrict__ head_scores, int H,
                                                        int S, int dh, int first_key, int col0,
                                                        int N, float scale_log2e) {
    constexpr int E = ElemTraits<T>::kPer16B;
    constexpr int cpr = 1 << LOG2_CPR;  // 16-byte pieces per key row
    constexpr int shift = LOG2_CPR;
    extern __shared__ __align__(16) unsigned char smem[];
    float *red = reinterpret_cast<float *>(smem);  // 16 floats
    float *qf = red + 16;                           // dh floats (dh <= 256)
    float *z = qf + 256;                            // n_keys floats

    const int h = blockIdx.x, bc = blockIdx.y;
    const int64_t head_row0 = ((int64_t)bc * H + h) * S;
    const T *qrow = q + head_row0 * dh;
    const unsigned char *kbase = reinterpret_cast<const unsigned char *>(k + (head_row0 + first_key) * dh);
    const int n_keys = S - first_key;
    const int tid = threadIdx.x;

    const int total = n_keys << shift;  // 16-byte pieces in the key block
    uint4 raw[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
        // clamped, not predicated: the loads of a batch stay independent of each other; what a
        // thread past the end fetched is dropped where the logits are filed
        const int p = min(u * 256 + tid, total - 1);
        raw[u] = load16_stream(kbase, (int64_t)p * 16);
    }
    for (int e = tid; e < dh; e += 256) qf[e] = load_elem<T>(qrow + e) * scale_log2e;
    __syncthreads();
    float qreg[E];
    const int piece = tid & (cpr - 1);
#pragma unroll
    for (int e = 0; e < E; ++e) qreg[e] = qf[piece * E + e];

    for (int base = 0; base < total; base += 256 * UNR) {
        uint4 nxt[UNR];
        if (base + 256 * UNR < total) {
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const int p = min(base + 256 * UNR + u * 256 + tid, total - 1);
                nxt[u] = load16_stream(kbase, (int64_t)p * 16);
            }
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int p = base + u * 256 + tid;
            float kv[E];
            unpack16<T>(raw[u], kv);
            float part = 0.f;
#pragma unroll
            for (int e = 0; e < E; ++e) part = fmaf(kv[e], qreg[e], part);
            part = group_sum<cpr>(part);
            if (piece == 0 && p < total) z[p >> shift] = part;
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) raw[u] = nxt[u];
    }
    __syncthreads();

    // softmax with one exchange between the waves: every wave normalises against its own
    // maximum, posts (maximum, sum) and rescales by what the four pairs combine to
    float m = -INFINITY;
    for (int j = tid; j < n_keys; j += 256) m = fmaxf(m, z[j]);
    m = wave_max(m);
    float sum = 0.f;
    for (int j = tid; j < n_keys; j += 256) {
        const float e = __builtin_amdgcn_exp2f(z[j] - m);
        z[j] = e;  // read again below by this same thread only
        sum += e;
    }
    sum = wave_sum(sum);
    if (lane_id() == 0) {
        red[wave_id()] = m;
        red[4 + wave_id()] = sum;
    }
    __syncthreads();
    const float mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    float denom = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) denom += red[4 + w] * __builtin_amdgcn_exp2f(red[w] - mx);
    // a wave without keys posted (-inf, 0): its term is 0 * 0
    const float f = __builtin_amdgcn_exp2f(m - mx) / denom;
    float *out = head_scores + ((int64_t)bc * H + h) * N;
    for (int j = tid; j < n_keys; j += 256)
        if (j >= col0 && j - col0 < N) out[j - col0] = z[j] * f;
}

// ---------------------------------------------------------------------------
// Mean attention received, on the matrix cores.
// ---------------------------------------------------------------------------
constexpr int kMeanBlock = 128;  // rows (pass 1) / keys (pass 2) owned by a workgroup
// rows of the streamed operand per LDS stage (smaller for wide rows: static LDS <= 64 KB)
__host__ __device__ constexpr int mean_tile_rows(int nc) { return nc > 8 ? 32 : 64; }

// Stages ROWS rows of NC 32-byte chunks through registers into LDS.
template <int NC, int ROWS>
struct TileStage {
    static constexpr int kPiecesPerRow = NC * 2;
    static constexpr int kPieces = ROWS * kPiecesPerRow;
    static constexpr int kPerThread = (kPieces + 255) / 256;
    static constexpr int kStride = NC * 32 + 16;  // bytes, padded against bank conflicts
    static constexpr int kBytes = ROWS * kStride;
    uint4 regs[kPerThread];

    // rows [row0, row0+ROWS) of a [*, row_bytes] matrix at `base`.  The loads carry no
    // condition: a row >= row_end re-reads row row_end - 1 and a piece past the end of a row
    // re-reads the row's last piece.  What lands in LDS for them is finite data that the
    // consumers neutralise (rows past the end are masked or carry an infinite log-sum-exp; the
    // register-resident operand is zero in the bytes past the row).
    __device__ __forceinline__ void load(const void *base, int row0, int row_end, int row_bytes) {
#pragma unroll
        for (int it = 0; it < kPerThread; ++it) {
            const int p = min((int)threadIdx.x + it * 256, kPieces - 1);
            const int r = p / kPiecesPerRow;
            const int piece = p - r * kPiecesPerRow;
            const int row = min(row0 + r, row_end - 1);
            regs[it] = load16(base, (int64_t)row * row_bytes + min(piece * 16, row_bytes - 16));
        }
    }
    __device__ __forceinline__ void store(unsigned char *lds) const {
#pragma unroll
        for (int it = 0; it < kPerThread; ++it) {
            const int p = threadIdx.x + it * 256;
            const int r = p / kPiecesPerRow;
            const int piece = p - r * kPiecesPerRow;
            if (p < kPieces) *reinterpret_cast<uint4 *>(lds + r * kStride + piece * 16) = regs[it];
        }
    }
};

// work item -> (segment*head, block) with each XCD walking a contiguous range of
// items, so the workgroups resident on one XCD share one head's Q/K in its L2
__device__ __forceinline__ int xcd_contiguous_item(int total) {
    const int id = blockIdx.x;
    const int per = (total + 7) / 8;
    return (id & 7) * per + (id >> 3);
}

// Pass 1: lse2[i] = log2 sum_j 2^(sl2 * q_i . k_j) over the key domain.
template <typename T, int NC>
__global__ __launch_bounds__(256, 2) void mean_lse_kernel(const T *__restrict__ q,
                                                          const T *__restrict__ k,
                                                          float *__restrict__ lse, int n_heads_total,
                                                          int S, int dh, int row_first, int N,
                                                          int key_first, int n_keys, float sl2) {
    constexpr int kMeanTile = mean_tile_rows(NC);
    using Stage = TileStage<NC, kMeanTile>;
    __shared__ __align__(16) unsigned char lds[2][Stage::kBytes];
    const int nblk = (N + kMeanBlock - 1) / kMeanBlock;
    const int total = n_heads_total * nblk;
    const int item = xcd_contiguous_item(total);
    if (item >= total) return;
    const int bh = item / nblk, rb = item - bh * nblk;
    const int row_bytes = dh * (int)sizeof(T);
    const unsigned char *qbase =
        reinterpret_cast<const unsigned char *>(q) + ((int64_t)bh * S + row_first) * row_bytes;
    const unsigned char *kbase =
        reinterpret_cast<const unsigned char *>(k) + ((int64_t)bh * S + key_first) * row_bytes;

    const int lane = lane_id(), g = lane >> 5, w = wave_id();
    const int qrow = rb * kMeanBlock + w * 32 + (lane & 31);
    uint4 qfrag[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c)
        qfrag[c] = load16_guard(qbase, (int64_t)qrow * row_bytes + 32 * c + 16 * g,
                                qrow < N && 32 * c + 16 * g < row_bytes);

    float m_run = -INFINITY, l_run = 0.f;
    bool have_ref = false;
    Stage st;
    const int ntiles = (n_keys + kMeanTile - 1) / kMeanTile;
    st.load(kbase, 0, n_keys, row_bytes);
    st.store(lds[0]);
    __syncthreads();
    for (int t = 0; t < ntiles; ++t) {
        const unsigned char *cur = lds[t & 1];
        if (t + 1 < ntiles) st.load(kbase, (t + 1) * kMeanTile, n_keys, row_bytes);
#pragma unroll
        for (int sub = 0; sub < kMeanTile / 32; ++sub) {
            f32x16_t acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.f;
            const unsigned char *arow = cur + (sub * 32 + (lane & 31)) * Stage::kStride + 16 * g;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const uint4 a = *reinterpret_cast<const uint4 *>(arow + 32 * c);
                mma32_chunk<T>(acc, a, qfrag[c]);
            }
            // acc[r] = q_row(lane%32) . k_(key0 + acc_row(r)); mask the ragged tail
            const int key0 = t * kMeanTile + sub * 32;
            if (key0 + 32 > n_keys) {
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (key0 + acc_row(r) >= n_keys) acc[r] = -INFINITY;
            }
            // Lazy reference: exponentials are taken against a per-lane reference m_run that
            // is an actual logit of the row (so the sum is >= 1 and small terms may underflow
            // harmlessly) and is only raised when the partial sum threatens to overflow.  That
            // removes the per-element running max; the rescue path is rare.
            if (!have_ref) {
                float mx = -INFINITY;
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, acc[r]);
                if (mx > -INFINITY) {
                    m_run = mx * sl2;
                    have_ref = true;
                }
            }
            if (have_ref) {
                float add = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    add += __builtin_amdgcn_exp2f(fmaf(acc[r], sl2, -m_run));
                if (add < 0x1p100f) {
                    l_run += add;
                } else {  // a logit far above the reference: re-base on this tile's maximum
                    float mx = -INFINITY;
#pragma unroll
                    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, acc[r]);
                    const float m_new = fmaxf(m_run, mx * sl2);
                    add = 0.f;
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        add += __builtin_amdgcn_exp2f(fmaf(acc[r], sl2, -m_new));
                    l_run = l_run * __builtin_amdgcn_exp2f(m_run - m_new) + add;
                    m_run = m_new;
                }
            }
        }
        if (t + 1 < ntiles) st.store(lds[(t + 1) & 1]);
        __syncthreads();
    }
    // the two half-waves hold disjoint key subsets of the same query row
    const float m_o = __shfl_xor(m_run, 32, kWave), l_o = __shfl_xor(l_run, 32, kWave);
    const float M = fmaxf(m_run, m_o);
    float L = 0.f;
    if (m_run > -INFINITY) L += l_run * __builtin_amdgcn_exp2f(m_run - M);
    if (m_o > -INFINITY) L += l_o * __builtin_amdgcn_exp2f(m_o - M);
    if (g == 0 && qrow < N) lse[(int64_t)bh * N + qrow] = M + log2f(L);
}

// Pass 2: head_scores[j] = sum_i 2^(sl2 * q_i . k_j - lse2[i]) for patch keys j.
template <typename T, int NC>
__global__ __launch_bounds__(256, 2) void mean_colsum_kernel(const T *__restrict__ q,
                                                             const T *__restrict__ k,
                                                             const float *__restrict__ lse,
                                                             float *__restrict__ head_scores,
                                                             int n_heads_total, int S, int dh,
                                                             int row_first, int N, float sl2) {
    constexpr int kMeanTile = mean_tile_rows(NC);
    using Stage = TileStage<NC, kMeanTile>;
    __shared__ __align__(16) unsigned char lds[2][Stage::kBytes];
    __shared__ __align__(16) float lse_s[2][kMeanTile];
    const int nblk = (N + kMeanBlock - 1) / kMeanBlock;
    const int total = n_heads_total * nblk;
    const int item = xcd_contiguous_item(total);
    if (item >= total) return;
    const int bh = item / nblk, kb = item - bh * nblk;
    const int row_bytes = dh * (int)sizeof(T);
    // queries and keys are both the patch rows here
    const unsigned char *qbase =
        reinterpret_cast<const unsigned char *>(q) + ((int64_t)bh * S + row_first) * row_bytes;
    const unsigned char *kbase =
        reinterpret_cast<const unsigned char *>(k) + ((int64_t)bh * S + row_first) * row_bytes;
    const float *lse_h = lse + (int64_t)bh * N;

    const int lane = lane_id(), g = lane >> 5, w = wave_id();
    const int key = kb * kMeanBlock + w * 32 + (lane & 31);
    uint4 kfrag[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c)
        kfrag[c] = load16_guard(kbase, (int64_t)key * row_bytes + 32 * c + 16 * g,
                                key < N && 32 * c + 16 * g < row_bytes);

    float colsum = 0.f;
    Stage st;
    const int ntiles = (N + kMeanTile - 1) / kMeanTile;
    const int tid = threadIdx.x;
    float lse_reg = 0.f;
    st.load(qbase, 0, N, row_bytes);
    if (tid < kMeanTile) lse_reg = tid < N ? lse_h[tid] : INFINITY;
    st.store(lds[0]);
    if (tid < kMeanTile) lse_s[0][tid] = lse_reg;
    __syncthreads();
    for (int t = 0; t < ntiles; ++t) {
        const unsigned char *cur = lds[t & 1];
        const float *lcur = lse_s[t & 1];
        if (t + 1 < ntiles) {
            st.load(qbase, (t + 1) * kMeanTile, N, row_bytes);
            const int r = (t + 1) * kMeanTile + tid;
            if (tid < kMeanTile) lse_reg = r < N ? lse_h[r] : INFINITY;
        }
#pragma unroll
        for (int sub = 0; sub < kMeanTile / 32; ++sub) {
            f32x16_t acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.f;
            const unsigned char *arow = cur + (sub * 32 + (lane & 31)) * Stage::kStride + 16 * g;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const uint4 a = *reinterpret_cast<const uint4 *>(arow + 32 * c);
                mma32_chunk<T>(acc, a, kfrag[c]);
            }
            // acc[r] = q_(row0 + acc_row(r)) . k_key ; rows past N carry lse = +inf -> 0
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                const float4 l4 =
                    *reinterpret_cast<const float4 *>(lcur + sub * 32 + 8 * rg + 4 * g);
                colsum += __builtin_amdgcn_exp2f(fmaf(acc[4 * rg + 0], sl2, -l4.x));
                colsum += __builtin_amdgcn_exp2f(fmaf(acc[4 * rg + 1], sl2, -l4.y));
                colsum += __builtin_amdgcn_exp2f(fmaf(acc[4 * rg + 2], sl2, -l4.z));
                colsum += __builtin_amdgcn_exp2f(fmaf(acc[4 * rg + 3], sl2, -l4.w));
            }
        }
        if (t + 1 < ntiles) {
            st.store(lds[(t + 1) & 1]);
            if (tid < kMeanTile) lse_s[(t + 1) & 1][tid] = lse_reg;
        }
        __syncthreads();
    }
    colsum += __shfl_xor(colsum, 32, kWave);
    if (g == 0 && key < N) head_scores[(int64_t)bh * N + key] = colsum;
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
template <typename T>
static hipError_t launch_score_cls_t(const ScoreArgs &a, hipStream_t s) {
    const int first_key = a.domain_all ? 0 : 1;
    const int n_keys = a.S - first_key;
    const size_t smem = (16 + 256 + (size_t)n_keys) * sizeof(float);
    if (smem > 64 * 1024) {
        hipError_t e =
            hipFuncSetAttribute(reinterpret_cast<const void *>(score_cls_generic_kernel<T>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
    }
    dim3 grid(a.H, a.BC);
    const int cpr = a.dh / ElemTraits<T>::kPer16B;
    // 16 pieces per thread and batch; 20 when that takes the whole key block in one batch (the
    // 577-row blocks of a 24 x 24 encoder with 128-byte heads: one memory round-trip less)
    const int64_t total = (int64_t)n_keys * cpr;
    // (only while every workgroup gets a CU to itself: the larger register set halves occupancy)
    const bool one_shot = total > 256 * 16 && total <= 256 * 20 && (int64_t)a.H * a.BC <= 256;
#define VSCAN_CLS_U(L, U)                                                                     \
    {                                                                                         \
        if (smem > 64 * 1024) {                                                               \
            hipError_t e = hipFuncSetAttribute(                                               \
                reinterpret_cast<const void *>(score_cls_kernel<T, L, U>),                    \
                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);                       \
            if (e != hipSuccess) return e;                                                    \
        }                                                                                     \
        hipLaunchKernelGGL((score_cls_kernel<T, L, U>), grid, dim3(256), smem, s,             \
                           (const T *)a.q, (const T *)a.k, a.head_scores, a.H, a.S, a.dh,     \
                           first_key, 1 - first_key, a.N, a.scale * 1.4426950408889634f);     \
        return hipGetLastError();                                                             \
    }
#define VSCAN_CLS(L)                                                                          \
    case L:                                                                                   \
        if (one_shot) VSCAN_CLS_U(L, 20)                                                      \
        VSCAN_CLS_U(L, 16)
    if ((cpr & (cpr - 1)) == 0) {
        switch (__builtin_ctz(cpr)) {
            VSCAN_CLS(0) VSCAN_CLS(1) VSCAN_CLS(2) VSCAN_CLS(3) VSCAN_CLS(4) VSCAN_CLS(5)
            VSCAN_CLS(6)
        }
    }
#undef VSCAN_CLS
#undef VSCAN_CLS_U
    {
        hipLaunchKernelGGL(score_cls_generic_kernel<T>, grid, dim3(256), smem, s, (const T *)a.q,
                           (const T *)a.k, a.head_scores, a.H, a.S, a.dh, first_key,
                           1 - first_key, a.N, a.scale * 1.4426950408889634f);
    }
    return hipGetLastError();
}

hipError_t launch_score_cls(const ScoreArgs &a, hipStream_t s) {
    return a.is_bf16 ? launch_score_cls_t<bf16_t>(a, s) : launch_score_cls_t<float>(a, s);
}

template <typename T, int NC>
static hipError_t launch_score_mean_nc(const ScoreArgs &a, hipStream_t s, int pass) {
    const int row_first = a.has_cls;
    const int key_first = a.domain_all ? 0 : a.has_cls;
    const int n_keys = a.S - key_first;
    const int nblk = (a.N + kMeanBlock - 1) / kMeanBlock;
    const int total = a.BC * a.H * nblk;
    const int grid = ((total + 7) / 8) * 8;
    const float sl2 = a.scale * 1.4426950408889634f;
    if (pass == 1)
        hipLaunchKernelGGL((mean_lse_kernel<T, NC>), dim3(grid), dim3(256), 0, s, (const T *)a.q,
                           (const T *)a.k, a.lse, a.BC * a.H, a.S, a.dh, row_first, a.N, key_first,
                           n_keys, sl2);
    else
        hipLaunchKernelGGL((mean_colsum_kernel<T, NC>), dim3(grid), dim3(256), 0, s,
                           (const T *)a.q, (const T *)a.k, a.lse, a.head_scores, a.BC * a.H, a.S,
                           a.dh, row_first, a.N, sl2);
    return hipGetLastError();
}

template <typename T>
static hipError_t launch_score_mean_t(const ScoreArgs &a, hipStream_t s, int pass) {
    const int nc = (a.dh * (int)sizeof(T) + 31) / 32;
    if (nc <= 2) return launch_score_mean_nc<T, 2>(a, s, pass);
    if (nc <= 4) return launch_score_mean_nc<T, 4>(a, s, pass);
    if (nc <= 5) return launch_score_mean_nc<T, 5>(a, s, pass);
    if (nc <= 8) return launch_score_mean_nc<T, 8>(a, s, pass);
    if (nc <= 12) return launch_score_mean_nc<T, 12>(a, s, pass);
    if (nc <= 16) return launch_score_mean_nc<T, 16>(a, s, pass);
    return hipErrorInvalidValue;  // rows wider than 512 bytes are rejected by the ABI layer
}

hipError_t launch_score_mean_lse(const ScoreArgs &a, hipStream_t s) {
    return a.is_bf16 ? launch_score_mean_t<bf16_t>(a, s, 1) : launch_score_mean_t<float>(a, s, 1);
}
hipError_t launch_score_mean_colsum(const ScoreArgs &a, hipStream_t s) {
    return a.is_bf16 ? launch_score_mean_t<bf16_t>(a, s, 2) : launch_score_mean_t<float>(a, s, 2);
}

}  // namespace vscan
