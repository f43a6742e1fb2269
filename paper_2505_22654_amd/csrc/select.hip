// Token selection: per-window local top-k then global top-k (Sec. 4.1, Eq. 2-3
// and the footnote on local priority), and the stage-2 top-k (Sec. 4.2).
//
// Thresholds tau / tau_w are realised as exact top-k counts with ties going to
// the lowest index.  No sort: a threshold key is found by radix / bitwise
// search on order-preserving integer keys held in LDS, then tokens are emitted
// in index order through prefix sums, which yields ascending lists directly.
#include "common.hpp"
#include "launch.hpp"

namespace vscan {

struct SelectSmem {
    uint32_t hist[256];
    int wsum[16];
    uint32_t bcast[4];
};

// Exclusive prefix count of `pred` over the block in thread order; `total` gets
// the block-wide count.  Two barriers.
__device__ __forceinline__ int block_excl_count(bool pred, int *wsum, int &total) {
    const uint64_t mask = __ballot(pred);
    const int pos = __popcll(mask & lanemask_lt());
    const int w = wave_id(), nw = blockDim.x / kWave;
    if (lane_id() == 0) wsum[w] = __popcll(mask);
    __syncthreads();
    int base = 0, tot = 0;
    for (int i = 0; i < nw; ++i) {
        const int c = wsum[i];
        if (i < w) base += c;
        tot += c;
    }
    __syncthreads();
    total = tot;
    return base + pos;
}

// Block-wide threshold search: among tokens j < n with flag[j] == 0 find the key T
// of the k-th largest (k >= 1, k <= number of such tokens).  Returns T; `need_eq`
// = how many tokens with key == T belong to the top k, `count_eq` = how many exist.
__device__ __forceinline__ uint32_t block_kth_key(const uint32_t *key, const uint8_t *flag, int n,
                                                  int k, SelectSmem &sm, int &need_eq,
                                                  int &count_eq) {
    uint32_t prefix = 0;
    int k_rem = k;
    const int tid = threadIdx.x;
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        if (tid < 256) sm.hist[tid] = 0;
        __syncthreads();
        for (int j = tid; j < n; j += blockDim.x) {
            if (flag[j]) continue;
            const uint32_t kk = key[j];
            if (pass == 0 || (kk >> (shift + 8)) == prefix) atomicAdd(&sm.hist[(kk >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (tid < kWave) {
            // lane l owns digits 255-4l .. 252-4l, walked from the top
            uint32_t c[4];
            uint32_t mine = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                c[i] = sm.hist[255 - (4 * tid + i)];
                mine += c[i];
            }
            uint32_t incl = mine;
#pragma unroll
            for (int o = 1; o < kWave; o <<= 1) {
                const uint32_t up = __shfl_up(incl, o, kWave);
                if (tid >= o) incl += up;
            }
            uint32_t above = incl - mine;  // tokens with a larger digit than any of mine
            if (above < (uint32_t)k_rem && (uint32_t)k_rem <= incl) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (above < (uint32_t)k_rem && (uint32_t)k_rem <= above + c[i]) {
                        sm.bcast[0] = 255 - (4 * tid + i);
                        sm.bcast[1] = (uint32_t)k_rem - above;
                        sm.bcast[2] = c[i];
                    }
                    above += c[i];
                }
            }
        }
        __syncthreads();
        prefix = (prefix << 8) | sm.bcast[0];
        k_rem = (int)sm.bcast[1];
        count_eq = (int)sm.bcast[2];
        __syncthreads();
    }
    need_eq = k_rem;
    return prefix;
}

// Marks (flag |= 2) the k best unflagged tokens by (key desc, index asc).
__device__ __forceinline__ void block_mark_topk(const uint32_t *key, uint8_t *flag, int n, int k,
                                                SelectSmem &sm) {
    if (k <= 0) return;
    int need_eq, count_eq;
    const uint32_t T = block_kth_key(key, flag, n, k, sm, need_eq, count_eq);
    if (need_eq == count_eq) {
        for (int j = threadIdx.x; j < n; j += blockDim.x)
            if (!flag[j] && key[j] >= T) flag[j] = 2;
        __syncthreads();
        return;
    }
    // ties at the threshold: take the first need_eq of them in index order
    int run = 0;
    for (int base = 0; base < n; base += blockDim.x) {
        const int j = base + threadIdx.x;
        const bool elig = j < n && !flag[j];
        const uint32_t kk = elig ? key[j] : 0u;
        const bool eq = elig && kk == T;
        int tot;
        const int rank = run + block_excl_count(eq, sm.wsum, tot);
        if (elig && (kk > T || (eq && rank < need_eq))) flag[j] = 2;
        run += tot;
    }
    __syncthreads();
}

// Wave-level top-kw inside one window of the token grid (rows [r0,r1), columns
// [c0,c1)): marks flag = 1.  All lanes of the wave must call it together.
__device__ __forceinline__ void wave_mark_window(const uint32_t *key, uint8_t *flag, int gw, int r0,
                                                 int r1, int c0, int c1, int kw) {
    const int wh = r1 - r0, ww = c1 - c0;
    int shift = 0;
    while ((1 << shift) < ww) ++shift;
    const int slots = wh << shift;
    const int steps = (slots + kWave - 1) / kWave;
    const int lane = lane_id();
    auto slot_key = [&](int st, int &idx) -> uint32_t {
        const int s = st * kWave + lane;
        const int rr = s >> shift, cc = s & ((1 << shift) - 1);
        const bool valid = rr < wh && cc < ww;
        idx = (r0 + rr) * gw + c0 + cc;
        return valid ? key[idx] : 0u;  // real keys are >= 1
    };
    uint32_t T = 0;
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t cand = T | (1u << bit);
        int cnt = 0;
        for (int st = 0; st < steps; ++st) {
            int idx;
            cnt += __popcll(__ballot(slot_key(st, idx) >= cand));
        }
        if (cnt >= kw) T = cand;
    }
    int cnt_gt = 0;
    for (int st = 0; st < steps; ++st) {
        int idx;
        cnt_gt += __popcll(__ballot(slot_key(st, idx) > T));
    }
    const int need_eq = kw - cnt_gt;
    int run = 0;
    for (int st = 0; st < steps; ++st) {
        int idx;
        const uint32_t kk = slot_key(st, idx);
        const bool eq = kk == T && kk != 0u;
        const uint64_t m = __ballot(eq);
        const int rank = run + __popcll(m & lanemask_lt());
        if (kk > T || (eq && rank < need_eq)) flag[idx] = 1;
        run += __popcll(m);
    }
}

__device__ __forceinline__ int ceil_div(int a, int b) { return (a + b - 1) / b; }

__global__ void encoder_select_kernel(EncSelectArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int N = a.gh * a.gw;
    SelectSmem &sm = *reinterpret_cast<SelectSmem *>(smem);
    uint32_t *keyg = reinterpret_cast<uint32_t *>(smem + sizeof(SelectSmem));
    uint32_t *keyl = a.head_local ? keyg + N : keyg;
    uint8_t *flag = reinterpret_cast<uint8_t *>((a.head_local ? keyl : keyg) + N);

    const int bc = blockIdx.x, b = bc / a.C, c = bc - b * a.C;
    const int tid = threadIdx.x;
    const int T_img = a.C * N;

    for (int j = tid; j < N; j += blockDim.x) {
        float sg = 0.f;
        for (int h = 0; h < a.H; ++h) sg += a.head_global[((int64_t)bc * a.H + h) * N + j];
        sg *= a.norm;
        keyg[j] = float_to_key(sg);
        if (a.scores_out) a.scores_out[(int64_t)b * T_img + (int64_t)c * N + j] = sg;
        if (a.head_local) {
            float sl = 0.f;
            for (int h = 0; h < a.H; ++h) sl += a.head_local[((int64_t)bc * a.H + h) * N + j];
            keyl[j] = float_to_key(sl * a.norm);
        }
        flag[j] = 0;
    }
    __syncthreads();

    // local scan: one wave per window
    if (a.kw > 0) {
        const int nW = a.wr * a.wc, nw = blockDim.x / kWave;
        for (int w = wave_id(); w < nW; w += nw) {
            const int wy = w / a.wc, wx = w - wy * a.wc;
            wave_mark_window(keyl, flag, a.gw, ceil_div(wy * a.gh, a.wr),
                             ceil_div((wy + 1) * a.gh, a.wr), ceil_div(wx * a.gw, a.wc),
                             ceil_div((wx + 1) * a.gw, a.wc), a.kw);
        }
    }
    __syncthreads();

    // global scan over what the local scan left
    block_mark_topk(keyg, flag, N, a.kg, sm);

    // emit ascending kept / dropped lists and seed the assignment array
    const int Kseg = a.wr * a.wc * a.kw + a.kg;
    const int K = a.C * Kseg, U = T_img - K;
    int run = 0;
    for (int base = 0; base < N; base += blockDim.x) {
        const int j = base + tid;
        const bool kept = j < N && flag[j] != 0;
        int tot;
        const int slot = run + block_excl_count(kept, sm.wsum, tot);
        if (j < N) {
            const int tok = c * N + j;
            if (kept) {
                const int s = c * Kseg + slot;
                a.kept_idx[(int64_t)b * K + s] = tok;
                a.best[(int64_t)b * T_img + tok] = (0xffffffffull << 32) | (uint32_t)~(uint32_t)s;
            } else {
                a.drop_idx[(int64_t)b * U + (int64_t)c * (N - Kseg) + (j - slot)] = tok;
                a.best[(int64_t)b * T_img + tok] = 0ull;
            }
        }
        run += tot;
    }
}

__global__ void llm_select_kernel(LlmSelectArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    SelectSmem &sm = *reinterpret_cast<SelectSmem *>(smem);
    uint32_t *key = reinterpret_cast<uint32_t *>(smem + sizeof(SelectSmem));
    uint8_t *flag = reinterpret_cast<uint8_t *>(key + a.V);
    const int b = blockIdx.x, tid = threadIdx.x, V = a.V;
    for (int j = tid; j < V; j += blockDim.x) {
        float s = 0.f;
        for (int g = 0; g < a.Hkv; ++g) s += a.part[((int64_t)b * a.Hkv + g) * V + j];
        s *= a.norm;
        key[j] = float_to_key(s);
        flag[j] = 0;
        if (a.scores_out) a.scores_out[(int64_t)b * V + j] = s;
    }
    __syncthreads();
    block_mark_topk(key, flag, V, a.keep, sm);
    int run = 0;
    for (int base = 0; base < V; base += blockDim.x) {
        const int j = base + tid;
        const bool kept = j < V && flag[j] != 0;
        int tot;
        const int slot = run + block_excl_count(kept, sm.wsum, tot);
        if (kept) a.kept_idx[(int64_t)b * a.keep + slot] = j;
        run += tot;
    }
}

// ---------------------------------------------------------------------------
// Small segments (N <= 1024): one thread per token, ranks by direct counting.
// Every loop runs over LDS with independent (pipelined) broadcast reads and there
// is no serial search, which is what matters when the whole call is a few
// microseconds long.  rank(j) = #{i : (key_i, -i) > (key_j, -j)}; a token is kept
// when its rank is below the budget, which is exactly top-k with ties to the
// lowest index.
// ---------------------------------------------------------------------------
constexpr int kSmallSelectMax = 1024;

// number of candidates that beat token j; cand[i] == 0 marks a non-candidate
__device__ __forceinline__ int count_better(const uint32_t *cand, int n4, uint32_t kj, int j) {
    int cnt = 0;
    const uint4 *c4 = reinterpret_cast<const uint4 *>(cand);
#pragma unroll 4
    for (int q = 0; q < n4; ++q) {
        const uint4 v = c4[q];
        const int i = 4 * q;
        cnt += (v.x > kj) || (v.x == kj && i < j);
        cnt += (v.y > kj) || (v.y == kj && i + 1 < j);
        cnt += (v.z > kj) || (v.z == kj && i + 2 < j);
        cnt += (v.w > kj) || (v.w == kj && i + 3 < j);
    }
    return cnt;
}

// slot of every kept token in thread (= token) order; two barriers
__device__ __forceinline__ int block_slot(bool kept, int *wsum) {
    int tot;
    return block_excl_count(kept, wsum, tot);
}

__global__ __launch_bounds__(1024) void encoder_select_small_kernel(EncSelectArgs a) {
    __shared__ __align__(16) uint32_t keyl[kSmallSelectMax];
    __shared__ __align__(16) uint32_t cand[kSmallSelectMax];  // global-scan candidates
    __shared__ int wsum[16];
    const int N = a.gh * a.gw;
    const int bc = blockIdx.x, b = bc / a.C, c = bc - b * a.C;
    const int j = threadIdx.x;
    const int T_img = a.C * N;
    const bool live = j < N;

    uint32_t kg_key = 0, kl_key = 0;
    if (live) {
        float sg = 0.f, sl = 0.f;
        const float *hg = a.head_global + (int64_t)bc * a.H * N + j;
        for (int h = 0; h < a.H; ++h) sg += hg[(int64_t)h * N];
        sg *= a.norm;
        kg_key = float_to_key(sg);
        if (a.scores_out) a.scores_out[(int64_t)b * T_img + (int64_t)c * N + j] = sg;
        if (a.head_local) {
            const float *hl = a.head_local + (int64_t)bc * a.H * N + j;
            for (int h = 0; h < a.H; ++h) sl += hl[(int64_t)h * N];
            kl_key = float_to_key(sl * a.norm);
        } else {
            kl_key = kg_key;
        }
    }
    keyl[j] = kl_key;  // 0 past the end
    __syncthreads();

    // local scan: rank inside the token's own window
    bool local = false;
    if (live && a.kw > 0) {
        const int r = j / a.gw, col = j - r * a.gw;
        const int wy = r * a.wr / a.gh, wx = col * a.wc / a.gw;
        const int r0 = ceil_div(wy * a.gh, a.wr), r1 = ceil_div((wy + 1) * a.gh, a.wr);
        const int c0 = ceil_div(wx * a.gw, a.wc), c1 = ceil_div((wx + 1) * a.gw, a.wc);
        int cnt = 0;
        for (int rr = r0; rr < r1; ++rr)
            for (int cc = c0; cc < c1; ++cc) {
                const int i = rr * a.gw + cc;
                const uint32_t ki = keyl[i];
                cnt += (ki > kl_key) || (ki == kl_key && i < j);
            }
        local = cnt < a.kw;
    }
    cand[j] = (live && !local) ? kg_key : 0u;
    __syncthreads();

    // global scan over what the local scan left
    bool global = false;
    if (live && !local && a.kg > 0)
        global = count_better(cand, (N + 3) >> 2, kg_key, j) < a.kg;

    const bool kept = local || global;
    const int slot = block_slot(kept, wsum);
    if (live) {
        const int Kseg = a.wr * a.wc * a.kw + a.kg;
        const int K = a.C * Kseg, U = T_img - K;
        const int tok = c * N + j;
        if (kept) {
            const int sidx = c * Kseg + slot;
            a.kept_idx[(int64_t)b * K + sidx] = tok;
            a.best[(int64_t)b * T_img + tok] = (0xffffffffull << 32) | (uint32_t)~(uint32_t)sidx;
        } else {
            a.drop_idx[(int64_t)b * U + (int64_t)c * (N - Kseg) + (j - slot)] = tok;
            a.best[(int64_t)b * T_img + tok] = 0ull;
        }
    }
}

__global__ __launch_bounds__(1024) void llm_select_small_kernel(LlmSelectArgs a) {
    __shared__ __align__(16) uint32_t cand[kSmallSelectMax];
    __shared__ int wsum[16];
    const int b = blockIdx.x, j = threadIdx.x, V = a.V;
    const bool live = j < V;
    uint32_t key = 0;
    if (live) {
        float s = 0.f;
        const float *pp = a.part + (int64_t)b * a.Hkv * V + j;
        for (int g = 0; g < a.Hkv; ++g) s += pp[(int64_t)g * V];
        s *= a.norm;
        key = float_to_key(s);
        if (a.scores_out) a.scores_out[(int64_t)b * V + j] = s;
    }
    cand[j] = key;
    __syncthreads();
    const bool kept = live && a.keep > 0 && count_better(cand, (V + 3) >> 2, key, j) < a.keep;
    const int slot = block_slot(kept, wsum);
    if (kept) a.kept_idx[(int64_t)b * a.keep + slot] = j;
}

static size_t round16(size_t v) { return (v + 15) & ~(size_t)15; }

size_t encoder_select_lds_bytes(int N, int has_local) {
    return sizeof(SelectSmem) + (size_t)N * 4 * (has_local ? 2 : 1) + round16((size_t)N);
}
size_t llm_select_lds_bytes(int V) { return sizeof(SelectSmem) + (size_t)V * 4 + round16((size_t)V); }

hipError_t launch_encoder_select(const EncSelectArgs &a, hipStream_t s) {
    const int N = a.gh * a.gw;
    if (N <= kSmallSelectMax) {
        const int threads = ((N + 3) / 4 * 4 + kWave - 1) / kWave * kWave;
        hipLaunchKernelGGL(encoder_select_small_kernel, dim3(a.B * a.C), dim3(threads), 0, s, a);
        return hipGetLastError();
    }
    const size_t smem = encoder_select_lds_bytes(N, a.head_local != nullptr);
    if (smem > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(encoder_select_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
    }
    const int threads = N > 2048 ? 1024 : 256;
    hipLaunchKernelGGL(encoder_select_kernel, dim3(a.B * a.C), dim3(threads), smem, s, a);
    return hipGetLastError();
}

hipError_t launch_llm_select(const LlmSelectArgs &a, hipStream_t s) {
    if (a.V <= kSmallSelectMax) {
        const int threads = ((a.V + 3) / 4 * 4 + kWave - 1) / kWave * kWave;
        hipLaunchKernelGGL(llm_select_small_kernel, dim3(a.B), dim3(threads), 0, s, a);
        return hipGetLastError();
    }
    const size_t smem = llm_select_lds_bytes(a.V);
    if (smem > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(llm_select_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
    }
    const int threads = a.V > 2048 ? 1024 : 256;
    hipLaunchKernelGGL(llm_select_kernel, dim3(a.B), dim3(threads), smem, s, a);
    return hipGetLastError();
}

}  // namespace vscan
