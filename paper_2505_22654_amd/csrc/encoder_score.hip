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
#include <type_traits>

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
// Both passes for bf16 rows of up to 160 bytes, software-pipelined inside each wave.
//
// Measured on this GPU (issue rates in core cycles per wave instruction): v_fma / v_mul / v_add
// 4, v_exp_f32 8, a 32x32x16 matrix instruction occupies the matrix pipe for 32 and takes about
// 10 from the vector issue port.  A 32 x 32 tile of logits therefore costs 16 x (4 + 8 + 4) = 256
// cycles of vector work per lane against 160 cycles of matrix work (80-element rows): the
// vector ALU is the bound, and the matrix instructions have to be hidden under it.  A wave that
// multiplies, waits and then exponentiates leaves both pipes idle in turn, so here every wave
// keeps two accumulator sets: the matrix instructions of tile t+1 are issued while the
// exponentials of tile t run, and the LDS reads of tile t+2's operands are already under way.
//
// A workgroup (4 waves) owns 4 x 32 x HALVES resident rows, held in registers as matrix
// operands (pass 1: query rows, pass 2: key rows).  The other operand streams through LDS in
// stages of 128 rows (4 tiles), two stages in LDS, the next one in flight in registers: one
// workgroup barrier per 128 streamed rows.  Accumulator layout as in mma32_chunk: a lane owns
// resident row (lane % 32) of each half and 16 of the 32 streamed rows of a tile.
//   PASS 1: lse2[i] = log2 sum_j 2^(sl2 * q_i . k_j)      (resident i, streamed j)
//   PASS 2: head_scores[j] = sum_i 2^(sl2 * q_i . k_j - lse2[i])   (resident j, streamed i)
// In pass 2 the subtraction rides on the matrix cores: every streamed row carries one more
// 32-byte chunk holding -lse2[i] / sl2 as three bf16 pieces (24 significant bits: the fp32 value
// exactly), the resident operand holds ones against them, so the accumulator comes out as
// q_i . k_j - lse2[i] / sl2 and a logit costs multiply, exponential, add with no per-row
// operand to fetch.  Rows past the end carry -inf and contribute 2^-inf = 0.
// ---------------------------------------------------------------------------
constexpr int kPipeStageRows = 128;

// 16-byte loads from global memory straight into LDS (no pass through vector registers, no LDS
// write instruction): lane l's data lands 16*l bytes behind the wave-uniform LDS address.  Issued
// from inline assembly so that the compiler's wait-count bookkeeping does not see them - it would
// otherwise make every LDS read wait for them, whichever buffer they fill; the kernel waits for
// them itself (wait_direct_loads) before the barrier that publishes the stage.
__device__ __forceinline__ unsigned lds_byte_address(const void *p) {
    return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}
__device__ __forceinline__ void direct_load16(const void *src, unsigned lds_address) {
    // (M0 carries the LDS address.  It is a reserved register that compiler-generated code
    // loads right before each instruction that reads it, never keeps live across statements,
    // and that the kernels of this file use for nothing else.)
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"
                 :
                 : "s"(lds_address), "v"(src)
                 : "memory");
}
// every outstanding vector-memory load of this wave has arrived (vmcnt 0, the other counters
// left alone)
__device__ __forceinline__ void wait_direct_loads() { __builtin_amdgcn_s_waitcnt(0x0F70); }

template <int NC, int HALVES, int PASS>
__global__ __launch_bounds__(256, 2) void mean_pipe_kernel(
    const unsigned char *__restrict__ resident, const unsigned char *__restrict__ streamed,
    const float *__restrict__ lse_in, float *__restrict__ out, int n_heads_total, int S, int dh,
    int res_first, int n_res, int str_first, int n_str, float sl2) {
    constexpr int NCX = NC + (PASS == 2 ? 1 : 0);      // chunks per streamed row (pass 2: the lse chunk)
    // With an odd number of 32-byte chunks per row the unpadded row pitch serves the 16-byte
    // operand reads at 92 % of the LDS rate (measured; 25 % for an even number), and a stage
    // is then one contiguous block in memory and in LDS alike: it is fetched with direct loads.
    // The lse chunk of pass 2 lives in an array of its own (32-byte rows).  Otherwise: padded
    // rows (pitch 32 NCX + 16, conflict-free) staged through registers.
    constexpr bool DIRECT = (NC & 1) != 0;
    constexpr int STRIDE = DIRECT ? NC * 32 : NCX * 32 + 16;
    constexpr int PPR = NC * 2;                        // 16-byte pieces per streamed row in memory
    constexpr int RB = 4 * 32 * HALVES;                // resident rows per workgroup
    constexpr int NM = NCX * HALVES;                   // matrix instructions per tile
    constexpr int NL = 16 * HALVES;                    // logits per lane and tile
    static_assert(kPipeStageRows * PPR == 256 * NC, "NC pieces per thread and stage");
    __shared__ __align__(16) unsigned char lds[2][kPipeStageRows * STRIDE];
    __shared__ __align__(16) unsigned char lse_lds[DIRECT && PASS == 2 ? 2 : 1][DIRECT && PASS == 2 ? kPipeStageRows * 32 : 16];

    const int nblk = (n_res + RB - 1) / RB;
    const int total = n_heads_total * nblk;
    const int item = xcd_contiguous_item(total);
    if (item >= total) return;
    const int bh = item / nblk, blk = item - bh * nblk;
    const int row_bytes = dh * 2;
    const unsigned char *rbase = resident + ((int64_t)bh * S + res_first) * row_bytes;
    const unsigned char *sbase = streamed + ((int64_t)bh * S + str_first) * row_bytes;
    const float *lse_h = PASS == 2 ? lse_in + (int64_t)bh * n_str : nullptr;

    const int tid = threadIdx.x, lane = lane_id(), g = lane >> 5, w = wave_id();
    uint4 kf[HALVES][NC];
#pragma unroll
    for (int h = 0; h < HALVES; ++h) {
        const int row = blk * RB + (w * HALVES + h) * 32 + (lane & 31);
#pragma unroll
        for (int c = 0; c < NC; ++c)
            kf[h][c] = load16_guard(rbase, (int64_t)row * row_bytes + 32 * c + 16 * g,
                                    row < n_res && 32 * c + 16 * g < row_bytes);
    }
    // pass 2: the resident side of the extra chunk, three ones (bf16 0x3f80) in the lower half
    const uint4 ones = g == 0 ? make_uint4(0x3f803f80u, 0x00003f80u, 0u, 0u) : zero16();

    const int ntiles = (n_str + 31) >> 5;
    const int nstages = (n_str + kPipeStageRows - 1) / kPipeStageRows;

    // ---- staging of the streamed operand: thread t carries pieces t, t + 256, ... of a stage
    uint4 sreg[DIRECT ? 1 : NC];
    float lse_reg = 0.f;
    auto stage_load = [&](int s) {
#pragma unroll
        for (int it = 0; it < NC; ++it) {
            const int p = tid + it * 256;
            const int r = p / PPR, piece = p - r * PPR;
            // clamped, not predicated: rows past the end re-read the last row (finite data that
            // the consumers neutralise), pieces past the end of a row its last piece (the
            // resident operand is zero there)
            const int row = min(s * kPipeStageRows + r, n_str - 1);
            const int64_t off = (int64_t)row * row_bytes + min(piece * 16, row_bytes - 16);
            if constexpr (DIRECT) {
                // piece p of the stage goes to byte 16 p of the stage's buffer: the wave's 64
                // pieces of this round form one contiguous kilobyte
                direct_load16(sbase + off, __builtin_amdgcn_readfirstlane(lds_byte_address(
                                               lds[s & 1] + 16 * (it * 256 + w * kWave))));
            } else {
                sreg[it] = load16(sbase, off);
            }
        }
        if (PASS == 2 && tid < kPipeStageRows)
            lse_reg = lse_h[min(s * kPipeStageRows + tid, n_str - 1)];
    };
    const float inv_sl2 = 1.0f / sl2;
    auto stage_store = [&](int s) {
        unsigned char *dst = lds[s & 1];
        if constexpr (DIRECT) {
            wait_direct_loads();  // this wave's share of the stage is in LDS
        } else {
#pragma unroll
            for (int it = 0; it < NC; ++it) {
                const int p = tid + it * 256;
                const int r = p / PPR, piece = p - r * PPR;
                *reinterpret_cast<uint4 *>(dst + r * STRIDE + piece * 16) = sreg[it];
            }
        }
        if (PASS == 2 && tid < kPipeStageRows) {
            // -lse / sl2 as hi + mid + lo; each residual is exact in fp32 and the third piece
            // takes what is left of the 24 bits.  (Decided here, not where the value was
            // fetched: arithmetic right behind the load would make the wave wait for it.)
            uint4 x = zero16();
            if (s * kPipeStageRows + tid < n_str) {
                const float v = -lse_reg * inv_sl2;
                const uint32_t hi = f32_to_bf16_rne(v);
                const float r1 = v - __uint_as_float(hi << 16);
                const uint32_t mid = f32_to_bf16_rne(r1);
                const float r2 = r1 - __uint_as_float(mid << 16);
                x.x = hi | (mid << 16);
                x.y = f32_to_bf16_rne(r2);
            } else {
                x.x = 0xff80u;  // -inf
            }
            unsigned char *e = DIRECT ? lse_lds[s & 1] + tid * 32 : dst + tid * STRIDE + NC * 32;
            *reinterpret_cast<uint4 *>(e) = x;
            *reinterpret_cast<uint4 *>(e + 16) = zero16();
        }
    };

    u32x4_t fr[NCX];      // streamed operand of one tile in matrix-operand layout, refilled in place
    f32x16_t acc[2][HALVES];
    auto frag_ptr = [&](int t) {
        return lds[(t >> 2) & 1] + ((t & 3) * 32 + (lane & 31)) * STRIDE + 16 * g;
    };
    // chunk c of tile t in matrix-operand layout (`base` = frag_ptr(t))
    auto read_frag = [&](const unsigned char *base, int t, int c) {
        if (DIRECT && c == NC)  // the lse chunk of pass 2
            return *reinterpret_cast<const u32x4_t *>(lse_lds[(t >> 2) & 1] +
                                                      ((t & 3) * 32 + (lane & 31)) * 32 + 16 * g);
        return *reinterpret_cast<const u32x4_t *>(base + 32 * c);
    };
    auto resident_frag = [&](int h, int c) {
        union {
            uint4 u;
            bf16x8_t v;
        } x;
        x.u = c < NC ? kf[h][c < NC ? c : 0] : ones;
        return x.v;
    };

    float m_run[HALVES], l_run[HALVES], colsum[HALVES];
    bool have_ref[HALVES];
#pragma unroll
    for (int h = 0; h < HALVES; ++h) {
        m_run[h] = -INFINITY;
        l_run[h] = 0.f;
        colsum[h] = 0.f;
        have_ref[h] = false;
    }

    // One pipeline step: the vector work of tile t (accumulators `cur`); when MULT is set, the
    // matrix instructions of tile t + 1 (operands in `fr`, accumulators `nxt`) are issued in
    // between, and every operand chunk is refilled with tile t + 2's (REFILL) right after its
    // last use.  MASK: tile t is the ragged last tile of pass 1.
    auto step = [&](int t, f32x16_t(&cur)[HALVES], f32x16_t(&nxt)[HALVES], auto mult_tag,
                    auto refill_tag, auto mask_tag) {
        constexpr bool MULT = decltype(mult_tag)::value, REFILL = decltype(refill_tag)::value,
                       MASK = decltype(mask_tag)::value;
        float ref[HALVES], part[HALVES];
        if constexpr (PASS == 1) {
            if constexpr (MASK) {
#pragma unroll
                for (int h = 0; h < HALVES; ++h)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (t * 32 + acc_row(r) >= n_str) cur[h][r] = -INFINITY;
            }
            // Lazy reference: exponentials are taken against a per-lane reference that is an
            // actual logit of the row (so the sum is >= 1 and small terms may underflow
            // harmlessly) and is only raised when the partial sum threatens to overflow.
#pragma unroll
            for (int h = 0; h < HALVES; ++h) {
                if (!have_ref[h]) {
                    float mx = -INFINITY;
#pragma unroll
                    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, cur[h][r]);
                    if (mx > -INFINITY) {
                        m_run[h] = mx * sl2;
                        have_ref[h] = true;
                    }
                }
                ref[h] = have_ref[h] ? m_run[h] : 0.f;  // without a reference every logit is -inf
            }
        }
#pragma unroll
        for (int h = 0; h < HALVES; ++h) part[h] = 0.f;
        const unsigned char *next_frags = REFILL ? frag_ptr(t + 2) : nullptr;
        // Slot by slot: one matrix instruction, the LDS read that refills an operand chunk
        // after its last use, and a slice of tile t's logits (about three: forty cycles of
        // vector work, which is what one matrix instruction keeps its pipe busy for).  (Pinning
        // this order with scheduling groups, or tying the step's inputs to this point with
        // empty asm statements, measured the same as leaving the order to the compiler.)
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            if constexpr (MULT) {
                const int c = m / HALVES, h = m % HALVES;
                // (the first chunk starts from a constant zero: no registers to clear)
                const f32x16_t zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f,
                                       0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                nxt[h] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    __builtin_bit_cast(bf16x8_t, fr[c]), resident_frag(h, c), c == 0 ? zero : nxt[h],
                    0, 0, 0);
                if constexpr (REFILL) {
                    if (h == HALVES - 1) fr[c] = read_frag(next_frags, t + 2, c);
                }
            }
#pragma unroll
            for (int i = m * NL / NM; i < (m + 1) * NL / NM; ++i) {
                const int h = i / 16, r = i % 16;
                if constexpr (PASS == 1)
                    part[h] += __builtin_amdgcn_exp2f(fmaf(cur[h][r], sl2, -ref[h]));
                else
                    part[h] += __builtin_amdgcn_exp2f(cur[h][r] * sl2);
            }
        }
#pragma unroll
        for (int h = 0; h < HALVES; ++h) {
            if constexpr (PASS == 2) {
                colsum[h] += part[h];
            } else {
                if (part[h] < 0x1p100f) {
                    l_run[h] += part[h];
                } else {  // a logit far above the reference: re-base on this tile's maximum
                    float mx = -INFINITY;
#pragma unroll
                    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, cur[h][r]);
                    const float m_new = fmaxf(m_run[h], mx * sl2);
                    float add = 0.f;
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        add += __builtin_amdgcn_exp2f(fmaf(cur[h][r], sl2, -m_new));
                    l_run[h] = l_run[h] * __builtin_amdgcn_exp2f(m_run[h] - m_new) + add;
                    m_run[h] = m_new;
                }
            }
        }
        // keep the steps apart: left alone, the compiler gathers the matrix instructions of
        // several steps into one burst right behind the LDS reads they wait for
        __builtin_amdgcn_sched_barrier(0);
    };
    using yes = std::integral_constant<bool, true>;
    using no = std::integral_constant<bool, false>;

    // ---- prologue: stage 0 in LDS, stage 1 in flight, tile 0 multiplied, tile 1's operands read
    stage_load(0);
    stage_store(0);
    __syncthreads();
    if (nstages > 1) stage_load(1);
    {
        const unsigned char *f0 = frag_ptr(0);
#pragma unroll
        for (int c = 0; c < NCX; ++c) fr[c] = read_frag(f0, 0, c);
#pragma unroll
        for (int h = 0; h < HALVES; ++h) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[0][h][r] = 0.f;
#pragma unroll
            for (int c = 0; c < NCX; ++c)
                acc[0][h] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    __builtin_bit_cast(bf16x8_t, fr[c]), resident_frag(h, c), acc[0][h], 0, 0, 0);
        }
        if (ntiles > 1) {
            const unsigned char *f1 = frag_ptr(1);
#pragma unroll
            for (int c = 0; c < NCX; ++c) fr[c] = read_frag(f1, 1, c);
        }
    }
    __builtin_amdgcn_sched_barrier(0);

    const bool ragged = PASS == 1 && (n_str & 31) != 0;
    int t0 = 0;
    // Steady state, four tiles (one stage) per trip: every step here has a tile t + 2 to fetch
    // operands for and a tile t + 1 to multiply, so the body is straight-line code.
    for (; t0 + 6 <= ntiles; t0 += 4) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = t0 + j;
            if (j == 2) {
                // the next stage goes to LDS now (its loads were issued four tiles ago), and
                // the one after it takes over the staging registers
                const int s = t >> 2;
                stage_store(s + 1);
                __syncthreads();
                if (s + 2 < nstages) stage_load(s + 2);
                __builtin_amdgcn_sched_barrier(0);
            }
            step(t, acc[j & 1], acc[(j + 1) & 1], yes{}, yes{}, no{});
        }
    }
    // The last tiles: the same steps with their conditions spelled out.
    for (; t0 < ntiles; t0 += 4) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = t0 + j;
            if (t < ntiles) {
                if (j == 2) {
                    const int s = t >> 2;
                    if (s + 1 < nstages) {
                        stage_store(s + 1);
                        __syncthreads();
                        if (s + 2 < nstages) stage_load(s + 2);
                    }
                }
                if (t + 2 < ntiles) {
                    step(t, acc[j & 1], acc[(j + 1) & 1], yes{}, yes{}, no{});
                } else if (t + 1 < ntiles) {
                    step(t, acc[j & 1], acc[(j + 1) & 1], yes{}, no{}, no{});
                } else if (ragged) {
                    step(t, acc[j & 1], acc[(j + 1) & 1], no{}, no{}, yes{});
                } else {
                    step(t, acc[j & 1], acc[(j + 1) & 1], no{}, no{}, no{});
                }
            }
        }
    }

    // the two half-waves hold disjoint streamed rows of the same resident row
#pragma unroll
    for (int h = 0; h < HALVES; ++h) {
        const int row = blk * RB + (w * HALVES + h) * 32 + (lane & 31);
        if constexpr (PASS == 1) {
            const float m_o = __shfl_xor(m_run[h], 32, kWave), l_o = __shfl_xor(l_run[h], 32, kWave);
            const float M = fmaxf(m_run[h], m_o);
            float L = 0.f;
            if (m_run[h] > -INFINITY) L += l_run[h] * __builtin_amdgcn_exp2f(m_run[h] - M);
            if (m_o > -INFINITY) L += l_o * __builtin_amdgcn_exp2f(m_o - M);
            if (g == 0 && row < n_res) out[(int64_t)bh * n_res + row] = M + log2f(L);
        } else {
            const float c = colsum[h] + __shfl_xor(colsum[h], 32, kWave);
            if (g == 0 && row < n_res) out[(int64_t)bh * n_res + row] = c;
        }
    }
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
        static std::atomic<uint64_t> lds_allowed{0};  // one per element type
        hipError_t e = allow_large_lds(score_cls_generic_kernel<T>, lds_allowed);
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
            static std::atomic<uint64_t> lds_allowed{0};                                      \
            hipError_t e = allow_large_lds(score_cls_kernel<T, L, U>, lds_allowed);           \
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

// The pipelined form: bf16 rows of up to 160 bytes (head sizes up to 80).
template <int NC, int HALVES>
static hipError_t launch_mean_pipe(const ScoreArgs &a, hipStream_t s, int pass) {
    const int row_first = a.has_cls;
    const int key_first = a.domain_all ? 0 : a.has_cls;
    const int n_keys = a.S - key_first;
    constexpr int RB = 4 * 32 * HALVES;
    const int total = a.BC * a.H * ((a.N + RB - 1) / RB);
    const int grid = ((total + 7) / 8) * 8;
    const float sl2 = a.scale * 1.4426950408889634f;
    const unsigned char *q = reinterpret_cast<const unsigned char *>(a.q);
    const unsigned char *k = reinterpret_cast<const unsigned char *>(a.k);
    if (pass == 1)  // resident query rows (patch rows), streamed keys of the softmax domain
        hipLaunchKernelGGL((mean_pipe_kernel<NC, HALVES, 1>), dim3(grid), dim3(256), 0, s, q, k,
                           (const float *)nullptr, a.lse, a.BC * a.H, a.S, a.dh, row_first, a.N,
                           key_first, n_keys, sl2);
    else            // resident patch keys, streamed query rows (patch rows) with their lse
        hipLaunchKernelGGL((mean_pipe_kernel<NC, HALVES, 2>), dim3(grid), dim3(256), 0, s, k, q,
                           (const float *)a.lse, a.head_scores, a.BC * a.H, a.S, a.dh, row_first,
                           a.N, row_first, a.N, sl2);
    return hipGetLastError();
}

template <typename T>
static hipError_t launch_score_mean_t(const ScoreArgs &a, hipStream_t s, int pass) {
    const int nc = (a.dh * (int)sizeof(T) + 31) / 32;
    if constexpr (sizeof(T) == 2) {
        if (nc <= 2) return launch_mean_pipe<2, 2>(a, s, pass);
        if (nc <= 4) return launch_mean_pipe<4, 2>(a, s, pass);
        if (nc <= 5) return launch_mean_pipe<5, 2>(a, s, pass);
    }
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
