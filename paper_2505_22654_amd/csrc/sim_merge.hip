// Similarity-based token merging (Sec. 4.1 "Token Merging", Eq. 4).
//
//   kept_inv_norm   1 / max(||x_s||, eps) for every kept token
//   sim_argmax      for every dropped token u: argmax_s (x_s . x_u) / ||x_s|| over
//                   the image's kept tokens.  ||x_u|| is a positive per-token
//                   constant and cannot change the argmax, so it is never formed.
//                   A kept x dropped GEMM on the matrix cores; the epilogue folds
//                   each column into a packed (similarity key, ~slot) word and
//                   merges it with atomicMax, which is order-independent and puts
//                   ties on the lowest slot.
//   merge           Eq. 4: one workgroup per kept slot averages the slot's own
//                   token and its members in ascending token order (fixed order:
//                   no floating-point atomics, bit-reproducible).
#include "common.hpp"
#include "launch.hpp"

namespace vscan {

constexpr float kNormEps = 1e-12f;

template <typename T>
__global__ __launch_bounds__(256) void kept_inv_norm_kernel(const T *__restrict__ x,
                                                            const int32_t *__restrict__ kept_idx,
                                                            float *__restrict__ inv_norm, int BK,
                                                            int K, int T_img, int D) {
    constexpr int E = ElemTraits<T>::kPer16B;
    const int row = blockIdx.x * (blockDim.x / kWave) + wave_id();
    if (row >= BK) return;
    const int b = row / K;
    const int tok = min(max(kept_idx[row], 0), T_img - 1);  // never index outside the image
    const T *xr = x + ((int64_t)b * T_img + tok) * D;
    float ss = 0.f;
    for (int p = lane_id(); p * E < D; p += kWave) {
        const uint4 raw = *reinterpret_cast<const uint4 *>(xr + p * E);
        float v[E];
        unpack16<T>(raw, v);
#pragma unroll
        for (int e = 0; e < E; ++e) ss = fmaf(v[e], v[e], ss);
    }
    ss = wave_sum(ss);
    if (lane_id() == 0) inv_norm[row] = 1.0f / fmaxf(sqrtf(ss), kNormEps);
}

// ---------------------------------------------------------------------------
// kept x dropped similarity with fused argmax.
// Workgroup tile: (64*TM) kept slots x (64*TN) dropped tokens, 4 waves as 2 x 2,
// each wave TM x TN blocks of 32 x 32.  The feature axis is streamed through LDS
// in stages of KC 32-byte chunks, double-buffered, rows gathered by index.
// ---------------------------------------------------------------------------
template <typename T, int TM, int TN, int KC>
__global__ __launch_bounds__(256) void sim_argmax_kernel(const T *__restrict__ x,
                                                         const int32_t *__restrict__ kept_idx,
                                                         const int32_t *__restrict__ drop_idx,
                                                         const float *__restrict__ inv_norm,
                                                         unsigned long long *__restrict__ best,
                                                         int T_img, int D, int K, int U) {
    constexpr int BM = 64 * TM, BN = 64 * TN, ROWS = BM + BN;
    constexpr int PPR = KC * 2;                 // 16-byte pieces per row per stage
    constexpr int STRIDE = KC * 32 + 16;        // LDS row stride in bytes
    constexpr int PER_THREAD = ROWS * PPR / 256;
    static_assert(ROWS * PPR % 256 == 0, "tile must split evenly over 256 threads");
    __shared__ __align__(16) unsigned char lds[2][ROWS * STRIDE];

    const int b = blockIdx.z;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int tid = threadIdx.x, lane = lane_id(), g = lane >> 5;
    const int wm = wave_id() >> 1, wn = wave_id() & 1;
    const int row_bytes = D * (int)sizeof(T);
    const unsigned char *xb = reinterpret_cast<const unsigned char *>(x) + (int64_t)b * T_img * row_bytes;

    // source byte offset of each piece this thread stages (-1: row outside the problem)
    int64_t src[PER_THREAD];
#pragma unroll
    for (int it = 0; it < PER_THREAD; ++it) {
        const int p = tid + it * 256;
        const int r = p / PPR;
        int tok = -1;
        if (r < BM) {
            if (m0 + r < K) tok = kept_idx[(int64_t)b * K + m0 + r];
        } else {
            if (n0 + r - BM < U) tok = drop_idx[(int64_t)b * U + n0 + r - BM];
        }
        tok = min(tok, T_img - 1);  // indices come from device memory: stay inside the image
        src[it] = tok < 0 ? -1 : (int64_t)tok * row_bytes + (p - r * PPR) * 16;
    }
    uint4 regs[PER_THREAD];
    auto stage_load = [&](int stage) {
#pragma unroll
        for (int it = 0; it < PER_THREAD; ++it) {
            const int p = tid + it * 256;
            const int piece = p % PPR;
            const int col_byte = stage * KC * 32 + piece * 16;
            regs[it] = load16_guard(xb, src[it] + (int64_t)stage * KC * 32,
                                    src[it] >= 0 && col_byte < row_bytes);
        }
    };
    auto stage_store = [&](unsigned char *dst) {
#pragma unroll
        for (int it = 0; it < PER_THREAD; ++it) {
            const int p = tid + it * 256;
            const int r = p / PPR;
            *reinterpret_cast<uint4 *>(dst + r * STRIDE + (p - r * PPR) * 16) = regs[it];
        }
    };

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int nstages = (row_bytes + KC * 32 - 1) / (KC * 32);
    stage_load(0);
    stage_store(lds[0]);
    __syncthreads();
    for (int st = 0; st < nstages; ++st) {
        const unsigned char *cur = lds[st & 1];
        if (st + 1 < nstages) stage_load(st + 1);
        const unsigned char *arow = cur + (wm * 32 * TM + (lane & 31)) * STRIDE + 16 * g;
        const unsigned char *brow = cur + (BM + wn * 32 * TN + (lane & 31)) * STRIDE + 16 * g;
#pragma unroll
        for (int c = 0; c < KC; ++c) {
            uint4 af[TM], bf[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                af[i] = *reinterpret_cast<const uint4 *>(arow + i * 32 * STRIDE + 32 * c);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                bf[j] = *reinterpret_cast<const uint4 *>(brow + j * 32 * STRIDE + 32 * c);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) mma32_chunk<T>(acc[i][j], af[i], bf[j]);
        }
        if (st + 1 < nstages) stage_store(lds[(st + 1) & 1]);
        __syncthreads();
    }

    // epilogue: acc[i][j][r] = x_slot . x_token with
    //   slot  = m0 + (wm*TM + i)*32 + acc_row(r),  token column = n0 + (wn*TN + j)*32 + lane%32
    const float *inv_b = inv_norm + (int64_t)b * K;
    float invs[TM][16];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int slot = m0 + (wm * TM + i) * 32 + acc_row(r);
            invs[i][r] = slot < K ? inv_b[slot] : 0.f;
        }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        float best_v = -INFINITY;
        int best_s = -1;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int slot = m0 + (wm * TM + i) * 32 + acc_row(r);
                if (slot < K) {
                    const float v = acc[i][j][r] * invs[i][r];
                    // slots are visited in ascending order: strict > keeps the lowest on ties
                    if (best_s < 0 || v > best_v) {
                        best_v = v;
                        best_s = slot;
                    }
                }
            }
        unsigned long long packed =
            best_s < 0 ? 0ull
                       : (((unsigned long long)float_to_key(best_v)) << 32) |
                             (unsigned long long)(uint32_t)~(uint32_t)best_s;
        const unsigned long long other = __shfl_xor(packed, 32, kWave);
        if (other > packed) packed = other;
        const int col = n0 + (wn * TN + j) * 32 + (lane & 31);
        if (g == 0 && col < U && packed != 0ull) {
            const int tok = min(max(drop_idx[(int64_t)b * U + col], 0), T_img - 1);
            atomicMax(best + (int64_t)b * T_img + tok, packed);
        }
    }
}

// ---------------------------------------------------------------------------
// Eq. 4.  grid (K, B); each thread owns 16-byte pieces of the feature row.
// ---------------------------------------------------------------------------
template <typename T, int PIECES>
__global__ __launch_bounds__(256) void merge_kernel(const T *__restrict__ x,
                                                    const unsigned long long *__restrict__ best,
                                                    T *__restrict__ merged,
                                                    int32_t *__restrict__ assign_out, int T_img,
                                                    int D, int K) {
    constexpr int E = ElemTraits<T>::kPer16B;
    __shared__ int wsum[4];
    __shared__ int members[256];
    const int slot = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const unsigned long long *bb = best + (int64_t)b * T_img;
    const T *xb = x + (int64_t)b * T_img * D;
    const int npieces = D / E;

    float acc[PIECES][E];
#pragma unroll
    for (int p = 0; p < PIECES; ++p)
#pragma unroll
        for (int e = 0; e < E; ++e) acc[p][e] = 0.f;

    int count = 0;
    for (int base = 0; base < T_img; base += 256) {
        const int t = base + tid;
        const bool mine = t < T_img && (int)(~(uint32_t)(bb[t] & 0xffffffffull)) == slot;
        // ordered compaction of this chunk's members
        const uint64_t mask = __ballot(mine);
        const int pos = __popcll(mask & lanemask_lt());
        if (lane_id() == 0) wsum[wave_id()] = __popcll(mask);
        __syncthreads();
        int off = 0, tot = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            if (w < wave_id()) off += wsum[w];
            tot += wsum[w];
        }
        if (mine) {
            members[off + pos] = t;
            if (assign_out) assign_out[(int64_t)b * T_img + t] = slot;
        }
        __syncthreads();
        // rows are fetched four members at a time and added in member order
        for (int m = 0; m < tot; m += 4) {
#pragma unroll
            for (int p = 0; p < PIECES; ++p) {
                const int piece = tid + p * 256;
                uint4 raw[4];
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    raw[i] = load16_guard(xb, ((int64_t)members[min(m + i, tot - 1)] * D +
                                               (int64_t)piece * E) * (int64_t)sizeof(T),
                                          m + i < tot && piece < npieces);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float v[E];
                    unpack16<T>(raw[i], v);
#pragma unroll
                    for (int e = 0; e < E; ++e) acc[p][e] += v[e];
                }
            }
        }
        count += tot;
        __syncthreads();
    }

    const float inv = 1.0f / (float)count;
    T *out = merged + ((int64_t)b * K + slot) * D;
#pragma unroll
    for (int p = 0; p < PIECES; ++p) {
        const int piece = tid + p * 256;
        if (piece < npieces) {
            uint4 o;
            if constexpr (sizeof(T) == 4) {
                o.x = __float_as_uint(acc[p][0] * inv);
                o.y = __float_as_uint(acc[p][1] * inv);
                o.z = __float_as_uint(acc[p][2] * inv);
                o.w = __float_as_uint(acc[p][3] * inv);
            } else {
                o.x = f32_to_bf16_rne(acc[p][0] * inv) | (f32_to_bf16_rne(acc[p][1] * inv) << 16);
                o.y = f32_to_bf16_rne(acc[p][2] * inv) | (f32_to_bf16_rne(acc[p][3] * inv) << 16);
                o.z = f32_to_bf16_rne(acc[p][4] * inv) | (f32_to_bf16_rne(acc[p][5] * inv) << 16);
                o.w = f32_to_bf16_rne(acc[p][6] * inv) | (f32_to_bf16_rne(acc[p][7] * inv) << 16);
            }
            *reinterpret_cast<uint4 *>(out + piece * E) = o;
        }
    }
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
template <typename T>
static hipError_t inv_norm_t(const MergeArgs &a, hipStream_t s) {
    const int rows = a.B * a.K;
    hipLaunchKernelGGL(kept_inv_norm_kernel<T>, dim3((rows + 3) / 4), dim3(256), 0, s,
                       (const T *)a.x, a.kept_idx, a.inv_norm, rows, a.K, a.T, a.D);
    return hipGetLastError();
}
hipError_t launch_kept_inv_norm(const MergeArgs &a, hipStream_t s) {
    return a.is_bf16 ? inv_norm_t<bf16_t>(a, s) : inv_norm_t<float>(a, s);
}

template <typename T, int TM, int TN>
static hipError_t sim_t(const MergeArgs &a, hipStream_t s) {
    constexpr int KC = 4;
    const int U = a.T - a.K;
    if (U <= 0) return hipSuccess;  // nothing was dropped: every token keeps its own slot
    dim3 grid((U + 64 * TN - 1) / (64 * TN), (a.K + 64 * TM - 1) / (64 * TM), a.B);
    hipLaunchKernelGGL((sim_argmax_kernel<T, TM, TN, KC>), grid, dim3(256), 0, s, (const T *)a.x,
                       a.kept_idx, a.drop_idx, a.inv_norm, (unsigned long long *)a.best, a.T, a.D,
                       a.K, U);
    return hipGetLastError();
}
hipError_t launch_sim_argmax(const MergeArgs &a, hipStream_t s) {
    // large problems amortise operand traffic with 128 x 128 tiles; small ones need
    // the workgroup count of 64 x 64 tiles to cover the chip
    const int U = a.T - a.K;
    const long tiles128 = (long)((U + 127) / 128) * ((a.K + 127) / 128) * a.B;
    const bool big = tiles128 >= 512;
    if (a.is_bf16) return big ? sim_t<bf16_t, 2, 2>(a, s) : sim_t<bf16_t, 1, 1>(a, s);
    return big ? sim_t<float, 2, 2>(a, s) : sim_t<float, 1, 1>(a, s);
}

template <typename T>
static hipError_t merge_t(const MergeArgs &a, hipStream_t s) {
    constexpr int E = ElemTraits<T>::kPer16B;
    const int npieces = a.D / E;
    dim3 grid(a.K, a.B);
#define VSCAN_MERGE(P)                                                                          \
    hipLaunchKernelGGL((merge_kernel<T, P>), grid, dim3(256), 0, s, (const T *)a.x,              \
                       (const unsigned long long *)a.best, (T *)a.merged, a.assign_out, a.T, a.D, \
                       a.K)
    if (npieces <= 256) VSCAN_MERGE(1);
    else if (npieces <= 512) VSCAN_MERGE(2);
    else if (npieces <= 1024) VSCAN_MERGE(4);
    else return hipErrorInvalidValue;  // wider rows are rejected by the ABI layer
#undef VSCAN_MERGE
    return hipGetLastError();
}
hipError_t launch_merge(const MergeArgs &a, hipStream_t s) {
    return a.is_bf16 ? merge_t<bf16_t>(a, s) : merge_t<float>(a, s);
}

}  // namespace vscan
