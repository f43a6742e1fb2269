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

// sum over heads of p[h * stride], added in head order; loads go out eight at a time so
// the sum costs a couple of memory round-trips instead of one per head
__device__ __forceinline__ float head_sum(const float *p, int heads, int stride) {
    float s = 0.f;
    for (int h0 = 0; h0 < heads; h0 += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = h0 + u < heads ? p[(int64_t)(h0 + u) * stride] : 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u];
    }
    return s;
}

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
        float sg = head_sum(a.head_global + (int64_t)bc * a.H * N + j, a.H, N);
        sg *= a.norm;
        keyg[j] = float_to_key(sg);
        if (a.scores_out) a.scores_out[(int64_t)b * T_img + (int64_t)c * N + j] = sg;
        if (a.head_local) {
            const float sl = head_sum(a.head_local + (int64_t)bc * a.H * N + j, a.H, N);
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
        float s = head_sum(a.part + (int64_t)b * a.Hkv * V + j, a.Hkv, V);
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
// Small segments (N <= 1024).  At this size a call lasts a few microseconds, so
// what counts is the length of the dependent instruction chain, not bandwidth:
// a top-k is found by ONE wave that holds its candidates' keys in registers and
// walks the 32 key bits from the top (one compare + ballot + popcount per register
// per bit, no LDS traffic and no barrier inside the search).  Windows are spread
// over the waves of the workgroup; the global scan is done by wave 0.
// ---------------------------------------------------------------------------
constexpr int kSmallSelectMax = 1024;

// Marks the k best of `nslots` slots; slot s -> (key, token) through `slot_fn`, which
// returns key 0 for a slot that is no candidate.  Slots are in ascending token order,
// so ties at the threshold go to the lowest token.  Called by a whole wave.
template <int NREG, typename SlotFn>
__device__ __forceinline__ void wave_topk_regs(SlotFn slot_fn, int nslots, int k, uint8_t *flag,
                                               uint8_t mark) {
    if (k <= 0) return;
    const int lane = lane_id();
    const int nreg = (nslots + kWave - 1) / kWave;  // <= NREG, wave-uniform
    uint32_t key[NREG];
    int idx[NREG];
#pragma unroll
    for (int r = 0; r < NREG; ++r) {
        key[r] = 0u;
        idx[r] = 0;
        const int sl = r * kWave + lane;
        if (r < nreg && sl < nslots) key[r] = slot_fn(sl, idx[r]);
    }
    // Counting is done per lane with vector compares and summed over the wave with DPP:
    // a compare whose result goes through a scalar register and a scalar popcount costs
    // an order of magnitude more per register on this hardware.  The serial part of a
    // step (reduce -> choose) dominates, so the threshold is built two bits at a time
    // from three independent candidate counts, and the walk stops as soon as some
    // candidate is reached by exactly k keys: the selected set is then already fixed.
    uint32_t T = 0;
    for (int shift = 30; shift >= 0; shift -= 2) {
        const uint32_t c1 = T | (1u << shift), c2 = T | (2u << shift), c3 = T | (3u << shift);
        int n1 = 0, n2 = 0, n3 = 0;  // registers past the last slot hold key 0 and never count
#pragma unroll
        for (int r = 0; r < NREG; ++r) {
            n1 += key[r] >= c1;
            n2 += key[r] >= c2;
            n3 += key[r] >= c3;
        }
        const int packed = wave_sum_dpp(n1 | (n2 << 16));
        const int t3 = wave_sum_dpp(n3);
        const int t1 = packed & 0xffff, t2 = packed >> 16;
        if (t3 >= k) {
            T = c3;
            if (t3 == k) break;
        } else if (t2 >= k) {
            T = c2;
            if (t2 == k) break;
        } else if (t1 >= k) {
            T = c1;
            if (t1 == k) break;
        }
    }
    int c_gt = 0, c_eq = 0;
#pragma unroll
    for (int r = 0; r < NREG; ++r) {
        c_gt += key[r] > T;
        c_eq += key[r] == T;
    }
    const int need_eq = k - wave_sum_dpp(c_gt);
    if (wave_sum_dpp(c_eq) == need_eq) {  // no tie straddles the boundary
#pragma unroll
        for (int r = 0; r < NREG; ++r)
            if (key[r] >= T) flag[idx[r]] = mark;  // T >= 1, so key 0 never passes
        return;
    }
    int run = 0;
#pragma unroll
    for (int r = 0; r < NREG; ++r)
        if (r < nreg) {
            const bool eq = key[r] == T;
            const uint64_t m = __ballot(eq);
            const int rank = run + __popcll(m & lanemask_lt());
            if (key[r] > T || (eq && rank < need_eq)) flag[idx[r]] = mark;
            run += __popcll(m);
        }
}

template <int NREG_W, int NREG_G>
__global__ __launch_bounds__(1024) void encoder_select_small_kernel(EncSelectArgs a) {
    __shared__ uint32_t keyl[kSmallSelectMax];
    __shared__ uint32_t keyg[kSmallSelectMax];
    __shared__ uint8_t flag[kSmallSelectMax];
    __shared__ int wsum[16];
    const int N = a.gh * a.gw;
    const int bc = blockIdx.x, b = bc / a.C, c = bc - b * a.C;
    const int j = threadIdx.x;
    const int T_img = a.C * N;
    const bool live = j < N;

    if (live) {
        const float sg = head_sum(a.head_global + (int64_t)bc * a.H * N + j, a.H, N) * a.norm;
        const uint32_t kg_key = float_to_key(sg);
        keyg[j] = kg_key;
        if (a.scores_out) a.scores_out[(int64_t)b * T_img + (int64_t)c * N + j] = sg;
        keyl[j] = a.head_local
                      ? float_to_key(head_sum(a.head_local + (int64_t)bc * a.H * N + j, a.H, N) *
                                     a.norm)
                      : kg_key;
        flag[j] = 0;
    }
    __syncthreads();

    // local scan.  Small windows: every token counts the tokens of its own window that
    // beat it (a few dozen pipelined LDS reads, no serial search).  Large windows: one wave
    // per window searches the threshold, windows round-robin over the waves.
    if (NREG_W == 0) {
        if (live && a.kw > 0) {
            const int r = j / a.gw, col = j - r * a.gw;
            const int wy = r * a.wr / a.gh, wx = col * a.wc / a.gw;
            const int r0 = ceil_div(wy * a.gh, a.wr), r1 = ceil_div((wy + 1) * a.gh, a.wr);
            const int c0 = ceil_div(wx * a.gw, a.wc), c1 = ceil_div((wx + 1) * a.gw, a.wc);
            const uint32_t kj = keyl[j];
            int cnt = 0;
            for (int rr = r0; rr < r1; ++rr) {
                const int row0 = rr * a.gw;
#pragma unroll 4
                for (int cc = c0; cc < c1; ++cc) {
                    const int i = row0 + cc;
                    const uint32_t ki = keyl[i];
                    cnt += (ki > kj) || (ki == kj && i < j);
                }
            }
            if (cnt < a.kw) flag[j] = 1;
        }
    } else if (a.kw > 0) {
        const int nW = a.wr * a.wc, nw = blockDim.x / kWave;
        for (int w = wave_id(); w < nW; w += nw) {
            const int wy = w / a.wc, wx = w - wy * a.wc;
            const int r0 = ceil_div(wy * a.gh, a.wr), r1 = ceil_div((wy + 1) * a.gh, a.wr);
            const int c0 = ceil_div(wx * a.gw, a.wc), c1 = ceil_div((wx + 1) * a.gw, a.wc);
            const int wh = r1 - r0, ww = c1 - c0;
            int shift = 0;
            while ((1 << shift) < ww) ++shift;
            const int gw = a.gw;
            wave_topk_regs<(NREG_W > 0 ? NREG_W : 1)>(
                [&](int sl, int &idx) -> uint32_t {
                    const int rr = sl >> shift, cc = sl & ((1 << shift) - 1);
                    idx = (r0 + rr) * gw + c0 + cc;
                    return cc < ww ? keyl[idx] : 0u;
                },
                wh << shift, a.kw, flag, 1);
        }
    }
    __syncthreads();

    // global scan over what the local scan left
    if (wave_id() == 0)
        wave_topk_regs<NREG_G>(
            [&](int sl, int &idx) -> uint32_t {
                idx = sl;
                return flag[sl] ? 0u : keyg[sl];
            },
            N, a.kg, flag, 2);
    __syncthreads();

    const bool kept = live && flag[j] != 0;
    int tot;
    const int slot = block_excl_count(kept, wsum, tot);
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

template <int NREG>
__global__ __launch_bounds__(1024) void llm_select_small_kernel(LlmSelectArgs a) {
    __shared__ uint32_t key[kSmallSelectMax];
    __shared__ uint8_t flag[kSmallSelectMax];
    __shared__ int wsum[16];
    const int b = blockIdx.x, j = threadIdx.x, V = a.V;
    const bool live = j < V;
    if (live) {
        const float s = head_sum(a.part + (int64_t)b * a.Hkv * V + j, a.Hkv, V) * a.norm;
        key[j] = float_to_key(s);
        flag[j] = 0;
        if (a.scores_out) a.scores_out[(int64_t)b * V + j] = s;
    }
    __syncthreads();
    if (wave_id() == 0)
        wave_topk_regs<NREG>(
            [&](int sl, int &idx) -> uint32_t {
                idx = sl;
                return key[sl];
            },
            V, a.keep, flag, 1);
    __syncthreads();
    const bool kept = live && flag[j] != 0;
    int tot;
    const int slot = block_excl_count(kept, wsum, tot);
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
        int threads = (N + kWave - 1) / kWave * kWave;
        // registers a wave needs: the largest window (columns padded to a power of two)
        // and the whole segment for the global scan
        int wcols = 1;
        while (wcols < (a.gw + a.wc - 1) / a.wc) wcols <<= 1;
        const int win_slots = a.kw > 0 ? ((a.gh + a.wr - 1) / a.wr) * wcols : 0;
        const bool count_windows = win_slots <= 256;  // rank by counting inside small windows
        if (!count_windows) {  // one wave per window where that fits
            const int want = a.wr * a.wc * kWave;
            if (want > threads) threads = want < 1024 ? want : 1024;
        }
        const int nreg_g = (N + kWave - 1) / kWave;
        const dim3 grid(a.B * a.C), block(threads);
#define VSCAN_SEL(W, G) hipLaunchKernelGGL((encoder_select_small_kernel<W, G>), grid, block, 0, s, a)
        if (count_windows) {
            if (nreg_g <= 4) VSCAN_SEL(0, 4);
            else if (nreg_g <= 10) VSCAN_SEL(0, 10);
            else VSCAN_SEL(0, 16);
        } else {
            if (nreg_g <= 10) VSCAN_SEL(32, 10);
            else VSCAN_SEL(32, 16);
        }
#undef VSCAN_SEL
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
        const int threads = (a.V + kWave - 1) / kWave * kWave;
        if (threads <= 4 * kWave)
            hipLaunchKernelGGL(llm_select_small_kernel<4>, dim3(a.B), dim3(threads), 0, s, a);
        else
            hipLaunchKernelGGL(llm_select_small_kernel<16>, dim3(a.B), dim3(threads), 0, s, a);
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
