// Token selection: per-window local top-k then global top-k (Sec. 4.1, Eq. 2-3
// and the footnote on local priority), and the stage-2 top-k (Sec. 4.2).
//
// Thresholds tau / tau_w are realised as exact top-k counts with ties going to
// the lowest index.  No sort: scores become order-preserving integer keys, the
// key of the k-th best is found by a most-significant-bit-first search over keys
// held in REGISTERS, and tokens are emitted in index order through ballot prefix
// sums, which yields ascending lists directly.
//
// What shapes the code: one call handles a few hundred to a few thousand tokens
// per segment, so it is a chain of dependent steps, not a bandwidth problem.
// Measured on gfx950: a vector compare whose result goes through a scalar
// register and a scalar popcount costs ~14 ns per register, a taken scalar
// branch ~13 ns, a workgroup barrier a few hundred ns.  Hence: counting is done
// per lane with vector compares and summed with DPP row operations, the
// threshold is built two bits per step from three independent candidate counts,
// and the walk stops as soon as some candidate is reached by exactly k keys.
#include "common.hpp"
#include "launch.hpp"

namespace vscan {

// sum over heads of p[h * stride], added in head order
__device__ __forceinline__ float head_sum(const float *p, int heads, int stride) {
    // sixteen heads at a time; the head index is clamped, not predicated, so that the loads of a
    // batch are independent of each other and in flight together
    float s = 0.f;
    for (int h0 = 0; h0 < heads; h0 += 16) {
        float v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = p[(int64_t)min(h0 + u, heads - 1) * stride];
#pragma unroll
        for (int u = 0; u < 16; ++u) s += h0 + u < heads ? v[u] : 0.f;
    }
    return s;
}

// Sum over the first sixteen lanes of a wave (one DPP row); every lane gets it.
__device__ __forceinline__ int row0_sum_dpp(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, true);   // quad_perm [1,0,3,2]
    v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, true);   // quad_perm [2,3,0,1]
    v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xf, 0xf, true);  // row_half_mirror
    v += __builtin_amdgcn_update_dpp(0, v, 0x140, 0xf, 0xf, true);  // row_mirror
    return __builtin_amdgcn_readlane(v, 0);
}

struct SelectSmem {
    int wsum[16];
    alignas(16) int cnt[2][16][4];  // per-wave candidate counts of the block-wide search, double-buffered
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

// Rank of every flagged token among the flagged ones.  Each wave owns one contiguous run of
// tokens and walks it 64 at a time (consecutive lanes, consecutive tokens: byte reads of the flags
// without bank conflicts, coalesced writes in `emit`).  A first pass counts the wave's flagged
// tokens, the totals cross LDS once, and the second pass hands out ranks (ballot population
// counts, on the scalar unit): two barriers in all, whatever the length.  `cnts`: LDS, one int
// per wave, free for this use.  emit(j, flagged, rank) is called once for every j < n.
template <typename Emit>
__device__ __forceinline__ void ranked_walk(const uint8_t *flag, int n, int *cnts, Emit emit) {
    const int nw = blockDim.x / kWave, w = wave_id(), lane = lane_id();
    const int rounds = (n + nw * kWave - 1) / (nw * kWave);  // per wave
    const int first = w * rounds * kWave;
    int total;
    if (rounds == 1) {
        total = __popcll(__ballot(first + lane < n && flag[first + lane] != 0));
    } else {
        // the count needs no order: the run's bytes four at a time, lane l taking words l, l + 64,
        // ... (a handful of independent LDS reads instead of one dependent read per 64 tokens)
        const uint32_t *words = reinterpret_cast<const uint32_t *>(flag + first);  // first % 64 == 0
        int mine = 0;
        for (int d = lane; d < rounds * (kWave / 4); d += kWave) {
            const int inside = n - (first + 4 * d);  // bytes of this word that belong to the list
            if (inside > 0) {
                uint32_t x = words[d];  // the flags' LDS is padded to a multiple of 16 bytes
                if (inside < 4) x &= (1u << (8 * inside)) - 1u;
                // flags are 0, 1 or 2: adding 3 sets bit 2 of exactly the non-zero bytes
                mine += __popc(((x & 0x03030303u) + 0x03030303u) & 0x04040404u);
            }
        }
        total = wave_sum_dpp(mine);
    }
    if (lane == 0) cnts[w] = total;
    __syncthreads();
    int run = row0_sum_dpp(lane < w ? cnts[lane] : 0);  // at most 16 waves
    for (int r = 0; r < rounds; ++r) {
        const int j = first + r * kWave + lane;
        const bool f = j < n && flag[j] != 0;
        const uint64_t m = __ballot(f);
        if (j < n) emit(j, f, run + __popcll(m & lanemask_lt()));
        run += __popcll(m);
    }
    __syncthreads();
}

__device__ __forceinline__ int ceil_div(int a, int b) { return (a + b - 1) / b; }

// ---------------------------------------------------------------------------
// Wave-level top-k.  Marks the k best of `nslots` slots; slot s -> (key, token)
// through `slot_fn`, which returns key 0 for a slot that is no candidate (every
// real key is >= 1).  Slots are in ascending token order, so ties at the
// threshold go to the lowest token.  Called by a whole wave; k <= candidates.
// ---------------------------------------------------------------------------
template <int NREG, typename SlotFn>
__device__ __forceinline__ void wave_topk_regs(SlotFn slot_fn, int nslots, int k, uint8_t *flag,
                                               uint8_t mark) {
    if (k <= 0) return;
    const int lane = lane_id();
    uint32_t key[NREG];
    int idx[NREG];
#pragma unroll
    for (int r = 0; r < NREG; ++r) {
        key[r] = 0u;
        idx[r] = 0;
        const int sl = r * kWave + lane;
        if (sl < nslots) key[r] = slot_fn(sl, idx[r]);
    }
    // The candidates' keys share their leading bits (the scores of one segment span a few
    // binades), and so does the threshold, which lies between the smallest and the largest of
    // them: the search starts at the highest bit in which those two differ.
    uint32_t kmax = 0u, inv_min = 0u;
#pragma unroll
    for (int r = 0; r < NREG; ++r) {
        kmax = max(kmax, key[r]);
        if (key[r] != 0u) inv_min = max(inv_min, ~key[r]);
    }
    kmax = wave_umax_dpp(kmax);
    if (kmax == 0u) return;  // no candidate at all
    const uint32_t diff = kmax ^ ~wave_umax_dpp(inv_min);
    const int top = diff ? (31 - __clz(diff)) & ~1 : -2;  // first pair of bits to decide
    uint32_t T = top >= 30 ? 0u : (top < 0 ? kmax : (kmax >> (top + 2)) << (top + 2));
    for (int shift = top; shift >= 0; shift -= 2) {
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
    for (int r = 0; r < NREG; ++r) {
        const bool eq = key[r] == T;
        const uint64_t m = __ballot(eq);
        const int rank = run + __popcll(m & lanemask_lt());
        if (key[r] > T || (eq && rank < need_eq)) flag[idx[r]] = mark;
        run += __popcll(m);
    }
}

// ---------------------------------------------------------------------------
// Block-level top-k for candidate sets too large for one wave: slot s = r*threads + t
// sits in register r of thread t.  Each step every wave sums its own three candidate
// counts with DPP and posts them to LDS; one barrier later every thread adds the
// posted counts (double-buffered, so one barrier per step).  Called by the whole
// block; k <= candidates.
// ---------------------------------------------------------------------------
template <int NREG, typename SlotFn>
__device__ __forceinline__ void block_topk_regs(SlotFn slot_fn, int nslots, int k, uint8_t *flag,
                                                uint8_t mark, SelectSmem &sm) {
    if (k <= 0) return;
    const int tid = threadIdx.x, nt = blockDim.x, nw = nt / kWave, w = wave_id();
    uint32_t key[NREG];
    int idx[NREG];
#pragma unroll
    for (int r = 0; r < NREG; ++r) {
        key[r] = 0u;
        idx[r] = 0;
        const int sl = r * nt + tid;
        if (sl < nslots) key[r] = slot_fn(sl, idx[r]);
    }
    // a, b, c: this wave's counts, already the same in every lane (ballot population counts,
    // which the scalar unit adds up beside the vector compares).  One lane posts them; after the
    // barrier lane i reads wave i's row in one access and a DPP sum over the wave adds the rows.
    auto exchange = [&](int buf, int a, int b, int c, int &ta, int &tb, int &tc) {
        if (lane_id() == 0) *reinterpret_cast<int4 *>(sm.cnt[buf][w]) = make_int4(a, b, c, 0);
        __syncthreads();
        int4 row = make_int4(0, 0, 0, 0);
        if (lane_id() < nw) row = *reinterpret_cast<const int4 *>(sm.cnt[buf][lane_id()]);
        ta = row0_sum_dpp(row.x);
        tb = row0_sum_dpp(row.y);
        tc = row0_sum_dpp(row.z);
    };
    // As in the wave-level search: start at the highest bit in which the largest and the
    // smallest candidate differ (one exchange of per-wave maxima through LDS).
    uint32_t kmax = 0u, inv_min = 0u;
#pragma unroll
    for (int r = 0; r < NREG; ++r) {
        kmax = max(kmax, key[r]);
        if (key[r] != 0u) inv_min = max(inv_min, ~key[r]);
    }
    kmax = wave_umax_dpp(kmax);
    inv_min = wave_umax_dpp(inv_min);
    if (lane_id() == 0) {
        sm.cnt[0][w][0] = (int)kmax;
        sm.cnt[0][w][1] = (int)inv_min;
    }
    __syncthreads();
    for (int i = 0; i < nw; ++i) {
        kmax = max(kmax, (uint32_t)sm.cnt[0][i][0]);
        inv_min = max(inv_min, (uint32_t)sm.cnt[0][i][1]);
    }
    if (kmax == 0u) {  // no candidate at all (uniform over the block)
        __syncthreads();
        return;
    }
    const uint32_t diff = kmax ^ ~inv_min;
    const int top = diff ? (31 - __clz(diff)) & ~1 : -2;  // first pair of bits to decide
    uint32_t T = top >= 30 ? 0u : (top < 0 ? kmax : (kmax >> (top + 2)) << (top + 2));
    int buf = 1;  // buffer 0 was just read: the first exchange writes the other one
    for (int shift = top; shift >= 0; shift -= 2) {
        const uint32_t c1 = T | (1u << shift), c2 = T | (2u << shift), c3 = T | (3u << shift);
        int n1 = 0, n2 = 0, n3 = 0;
#pragma unroll
        for (int r = 0; r < NREG; ++r) {
            n1 += __popcll(__ballot(key[r] >= c1));
            n2 += __popcll(__ballot(key[r] >= c2));
            n3 += __popcll(__ballot(key[r] >= c3));
        }
        int t1, t2, t3;
        exchange(buf, n1, n2, n3, t1, t2, t3);
        buf ^= 1;
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
        c_gt += __popcll(__ballot(key[r] > T));
        c_eq += __popcll(__ballot(key[r] == T));
    }
    int t_gt, t_eq, unused;
    exchange(buf, c_gt, 0, c_eq, t_gt, unused, t_eq);
    const int need_eq = k - t_gt;
    if (t_eq == need_eq) {
#pragma unroll
        for (int r = 0; r < NREG; ++r)
            if (key[r] >= T) flag[idx[r]] = mark;
        __syncthreads();
        return;
    }
    __syncthreads();  // the prefix counts below reuse LDS that `exchange` may still be reading
    int run = 0;
#pragma unroll
    for (int r = 0; r < NREG; ++r) {  // slot order = (register, thread): ascending tokens
        const bool eq = key[r] == T;
        int tot;
        const int rank = run + block_excl_count(eq, sm.wsum, tot);
        if (key[r] > T || (eq && rank < need_eq)) flag[idx[r]] = mark;
        run += tot;
    }
    __syncthreads();
}

struct WindowGeom {
    int r0, c0, wh, ww, shift;  // slot s -> row r0 + (s >> shift), column c0 + (s & mask)
};
__device__ __forceinline__ WindowGeom window_geom(const EncSelectArgs &a, int w) {
    const int wy = w / a.wc, wx = w - wy * a.wc;
    WindowGeom g;
    g.r0 = ceil_div(wy * a.gh, a.wr);
    g.c0 = ceil_div(wx * a.gw, a.wc);
    g.wh = ceil_div((wy + 1) * a.gh, a.wr) - g.r0;
    g.ww = ceil_div((wx + 1) * a.gw, a.wc) - g.c0;
    g.shift = 0;
    while ((1 << g.shift) < g.ww) ++g.shift;
    return g;
}

// ---------------------------------------------------------------------------
// Encoder selection, one workgroup per segment.
//   WIN_MODE 0: every token ranks itself inside its own window by counting (windows of at
//               most 256 slots: a few dozen pipelined LDS reads, no serial search)
//   WIN_MODE 3: the same ranking for segments with one thread per token: keys are first copied
//               window by window, so that a token reads its rivals 16 bytes at a time, and
//               the window geometry comes from two small tables instead of divisions
//   WIN_MODE 1: one wave per window, wave_topk_regs<NREG_W>
//   WIN_MODE 2: windows one after the other, block_topk_regs<NREG_G>
// Global scan: wave 0 alone when the segment fits its registers (GLOBAL_WAVE), else the block.
// ---------------------------------------------------------------------------
template <int WIN_MODE, int NREG_W, bool GLOBAL_WAVE, int NREG_G>
__global__ __launch_bounds__(1024) void encoder_select_kernel(EncSelectArgs a, int win_pitch) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int N = a.gh * a.gw;
    SelectSmem &sm = *reinterpret_cast<SelectSmem *>(smem);
    uint32_t *keyg = reinterpret_cast<uint32_t *>(smem + sizeof(SelectSmem));
    uint32_t *keyl = a.head_local ? keyg + N : keyg;
    uint8_t *flag = reinterpret_cast<uint8_t *>((a.head_local ? keyl : keyg) + N);

    const int bc = blockIdx.x, b = bc / a.C, c = bc - b * a.C;
    const int tid = threadIdx.x, nt = blockDim.x;
    const int T_img = a.C * N;

    if (a.pre_key) {
        // large segment: head sums, keys and the local scan were done window by window by
        // encoder_select_local_kernel; what is left is the global scan and the lists
        // every thread's values requested at once (clamped positions): a loop of one load per
        // trip would be a chain of memory round-trips
        uint32_t kreg[NREG_G];
        uint8_t freg[NREG_G];
#pragma unroll
        for (int r = 0; r < NREG_G; ++r) {
            const int64_t j = (int64_t)bc * N + min(r * nt + tid, N - 1);
            kreg[r] = a.pre_key[j];
            freg[r] = a.pre_flag[j];
        }
#pragma unroll
        for (int r = 0; r < NREG_G; ++r) {
            const int j = r * nt + tid;
            if (j < N) {
                keyg[j] = kreg[r];
                flag[j] = freg[r];
            }
        }
    } else {
        for (int j = tid; j < N; j += nt) {
            const float sg = head_sum(a.head_global + (int64_t)bc * a.H * N + j, a.H, N) * a.norm;
            keyg[j] = float_to_key(sg);
            if (a.scores_out) a.scores_out[(int64_t)b * T_img + (int64_t)c * N + j] = sg;
            if (a.head_local)
                keyl[j] = float_to_key(head_sum(a.head_local + (int64_t)bc * a.H * N + j, a.H, N) *
                                       a.norm);
            flag[j] = 0;
        }
    }
    __syncthreads();

    // ---- local scan (Eq. 3) ----
    const int nW = a.wr * a.wc;
    if (a.kw > 0 && !a.pre_key) {
        if (WIN_MODE == 3) {
            // LDS behind the flags: the window-major keys (`win_pitch` slots per window, unused
            // slots zero: no real key is zero), then per grid row and per grid column the window
            // coordinate, the offset inside the window, and the window's extent along that axis.
            uint32_t *wk = reinterpret_cast<uint32_t *>(
                smem + (((size_t)(flag - smem) + N + 15) & ~(size_t)15));
            int *row_tab = reinterpret_cast<int *>(wk + nW * win_pitch);  // [gh][3]
            int *col_tab = row_tab + 3 * a.gh;                             // [gw][3]
            for (int i = tid; i < nW * win_pitch; i += nt) wk[i] = 0u;
            for (int i = tid; i < a.gh + a.gw; i += nt) {
                const bool is_row = i < a.gh;
                const int p = is_row ? i : i - a.gh;        // position along the axis
                const int n = is_row ? a.gh : a.gw, nwin = is_row ? a.wr : a.wc;
                const int wi = p * nwin / n;                // window coordinate of this position
                const int first = ceil_div(wi * n, nwin);
                int *t = (is_row ? row_tab : col_tab) + 3 * p;
                t[0] = wi;
                t[1] = p - first;
                t[2] = ceil_div((wi + 1) * n, nwin) - first;
            }
            __syncthreads();
            int w = 0, slot = 0;
            uint32_t kj = 0u;
            if (tid < N) {
                // tid / gw without an integer division: exact for tid < 2^20 (the half keeps the
                // product clear of the integer boundaries)
                const int r = (int)(((float)tid + 0.5f) * (1.0f / (float)a.gw));
                const int col = tid - r * a.gw;
                const int *rt = row_tab + 3 * r, *ct = col_tab + 3 * col;
                w = rt[0] * a.wc + ct[0];
                slot = rt[1] * ct[2] + ct[1];               // row-major inside the window
                kj = keyl[tid];
                wk[w * win_pitch + slot] = kj;
            }
            __syncthreads();
            if (tid < N) {
                // rank among the window's slots; row-major slot order is ascending token order,
                // which is what ties are broken by
                const uint4 *row = reinterpret_cast<const uint4 *>(wk + w * win_pitch);
                int cnt = 0;
                for (int i = 0; i < win_pitch / 4; ++i) {
                    const uint4 k4 = row[i];
                    const int s0 = 4 * i;
                    cnt += (k4.x > kj) || (k4.x == kj && s0 < slot);
                    cnt += (k4.y > kj) || (k4.y == kj && s0 + 1 < slot);
                    cnt += (k4.z > kj) || (k4.z == kj && s0 + 2 < slot);
                    cnt += (k4.w > kj) || (k4.w == kj && s0 + 3 < slot);
                }
                if (cnt < a.kw) flag[tid] = 1;
            }
        } else if (WIN_MODE == 0) {
            for (int j = tid; j < N; j += nt) {
                const int r = j / a.gw, col = j - r * a.gw;
                const WindowGeom g = window_geom(a, (r * a.wr / a.gh) * a.wc + col * a.wc / a.gw);
                const uint32_t kj = keyl[j];
                int cnt = 0;
                for (int rr = g.r0; rr < g.r0 + g.wh; ++rr) {
                    const int row0 = rr * a.gw;
#pragma unroll 4
                    for (int cc = g.c0; cc < g.c0 + g.ww; ++cc) {
                        const int i = row0 + cc;
                        const uint32_t ki = keyl[i];
                        cnt += (ki > kj) || (ki == kj && i < j);
                    }
                }
                if (cnt < a.kw) flag[j] = 1;
            }
        } else if (WIN_MODE == 1) {
            for (int w = wave_id(); w < nW; w += nt / kWave) {
                const WindowGeom g = window_geom(a, w);
                const int gw = a.gw;
                wave_topk_regs<NREG_W>(
                    [&](int sl, int &idx) -> uint32_t {
                        const int rr = sl >> g.shift, cc = sl & ((1 << g.shift) - 1);
                        idx = (g.r0 + rr) * gw + g.c0 + cc;
                        return cc < g.ww ? keyl[idx] : 0u;
                    },
                    g.wh << g.shift, a.kw, flag, 1);
            }
        } else {
            for (int w = 0; w < nW; ++w) {
                const WindowGeom g = window_geom(a, w);
                const int gw = a.gw;
                block_topk_regs<NREG_G>(
                    [&](int sl, int &idx) -> uint32_t {
                        const int rr = sl >> g.shift, cc = sl & ((1 << g.shift) - 1);
                        idx = (g.r0 + rr) * gw + g.c0 + cc;
                        return cc < g.ww ? keyl[idx] : 0u;
                    },
                    g.wh << g.shift, a.kw, flag, 1, sm);
            }
        }
    }
    __syncthreads();

    // ---- global scan over what the local scan left (Eq. 2 + footnote) ----
    auto global_slot = [&](int sl, int &idx) -> uint32_t {
        idx = sl;
        return flag[sl] ? 0u : keyg[sl];
    };
    if (GLOBAL_WAVE) {
        if (wave_id() == 0) wave_topk_regs<NREG_G>(global_slot, N, a.kg, flag, 2);
        __syncthreads();
    } else {
        block_topk_regs<NREG_G>(global_slot, N, a.kg, flag, 2, sm);
    }

    // ---- ascending kept / dropped lists; seed the assignment words ----
    const int Kseg = nW * a.kw + a.kg;
    const int K = a.C * Kseg, U = T_img - K;
    // (the keys are no longer needed: their LDS holds the per-round counts of the walk)
    __syncthreads();
    ranked_walk(flag, N, reinterpret_cast<int *>(keyg), [&](int j, bool kept, int slot) {
        const int tok = c * N + j;
        if (kept) {
            const int s = c * Kseg + slot;
            a.kept_idx[(int64_t)b * K + s] = tok;
            a.best[(int64_t)b * T_img + tok] = (0xffffffffull << 32) | (uint32_t)~(uint32_t)s;
        } else {
            a.drop_idx[(int64_t)b * U + (int64_t)c * (N - Kseg) + (j - slot)] = tok;
            a.best[(int64_t)b * T_img + tok] = 0ull;
        }
    });
}

// Large segments, first half: one workgroup per window (or per 1024 tokens when there is no local
// scan).  A single workgroup that walks a 16384-token segment spends most of its time fetching
// H values per token at the rate one compute unit can take them; here every window's tokens are
// summed over the heads, turned into keys and ranked inside the window (by counting: window
// slots in row-major order are ascending token indices, which is what ties are broken by) by a
// workgroup of its own.  Outputs: the global-scan key and the local-scan flag of every token.
__global__ __launch_bounds__(1024) void encoder_select_local_kernel(EncSelectArgs a,
                                                                   uint32_t *__restrict__ key_out,
                                                                   uint8_t *__restrict__ flag_out) {
    __shared__ __align__(16) uint32_t wk[1024];
    const int N = a.gh * a.gw, T_img = a.C * N;
    const int bc = blockIdx.y, b = bc / a.C, c = bc - b * a.C;
    const int tid = threadIdx.x;
    int j = -1, slots = 0;
    if (a.kw > 0) {
        const WindowGeom g = window_geom(a, blockIdx.x);
        slots = g.wh * g.ww;
        if (tid < slots) {
            const int rr = tid / g.ww, cc = tid - rr * g.ww;
            j = (g.r0 + rr) * a.gw + g.c0 + cc;
        }
    } else if (blockIdx.x * 1024 + tid < N) {
        j = blockIdx.x * 1024 + tid;
    }
    uint32_t kl = 0u;
    if (j >= 0) {
        const float sg = head_sum(a.head_global + (int64_t)bc * a.H * N + j, a.H, N) * a.norm;
        const uint32_t kg = float_to_key(sg);
        key_out[(int64_t)bc * N + j] = kg;
        if (a.scores_out) a.scores_out[(int64_t)b * T_img + (int64_t)c * N + j] = sg;
        kl = a.head_local
                 ? float_to_key(head_sum(a.head_local + (int64_t)bc * a.H * N + j, a.H, N) * a.norm)
                 : kg;
    }
    if (a.kw <= 0) {
        if (j >= 0) flag_out[(int64_t)bc * N + j] = 0;
        return;
    }
    wk[tid] = kl;  // threads past the window hold key 0, below every real key
    __syncthreads();
    if (j < 0) return;
    int cnt = 0;
    const uint4 *row = reinterpret_cast<const uint4 *>(wk);
    for (int i = 0; i < (slots + 3) / 4; ++i) {
        const uint4 k4 = row[i];
        const int s0 = 4 * i;
        cnt += (k4.x > kl) || (k4.x == kl && s0 < tid);
        cnt += (k4.y > kl) || (k4.y == kl && s0 + 1 < tid);
        cnt += (k4.z > kl) || (k4.z == kl && s0 + 2 < tid);
        cnt += (k4.w > kl) || (k4.w == kl && s0 + 3 < tid);
    }
    flag_out[(int64_t)bc * N + j] = cnt < a.kw ? 1 : 0;
}

// Stage-2 selection, one workgroup per sequence.
template <bool GLOBAL_WAVE, int NREG>
__global__ __launch_bounds__(1024) void llm_select_kernel(LlmSelectArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    SelectSmem &sm = *reinterpret_cast<SelectSmem *>(smem);
    uint32_t *key = reinterpret_cast<uint32_t *>(smem + sizeof(SelectSmem));
    uint8_t *flag = reinterpret_cast<uint8_t *>(key + a.V);
    const int b = blockIdx.x, tid = threadIdx.x, nt = blockDim.x;
    // ragged batch: this sequence's own span and budget; a.V and a.keep stay the strides
    const int V = a.meta ? a.meta[b].vis_len : a.V;
    const int keep = a.meta ? a.meta[b].keep : a.keep;
    if (GLOBAL_WAVE) {
        for (int j = tid; j < V; j += nt) {  // one token per thread
            const float s = head_sum(a.part + (int64_t)b * a.Hkv * a.V + j, a.Hkv, a.V) * a.norm;
            key[j] = float_to_key(s);
            flag[j] = 0;
            if (a.scores_out) a.scores_out[(int64_t)b * a.V + j] = s;
        }
    } else {
        // several tokens per thread: the head values of all of them are requested together,
        // a few heads at a time (clamped positions), and added in head order as head_sum does
        constexpr int HB = NREG <= 4 ? 8 : NREG <= 16 ? 2 : 1;
        float acc[NREG];
#pragma unroll
        for (int r = 0; r < NREG; ++r) acc[r] = 0.f;
        const float *pb = a.part + (int64_t)b * a.Hkv * a.V;
        for (int h0 = 0; h0 < a.Hkv; h0 += HB) {
            float v[NREG][HB];
#pragma unroll
            for (int r = 0; r < NREG; ++r)
#pragma unroll
                for (int u = 0; u < HB; ++u)
                    v[r][u] = pb[(int64_t)min(h0 + u, a.Hkv - 1) * a.V + min(r * nt + tid, V - 1)];
#pragma unroll
            for (int r = 0; r < NREG; ++r)
#pragma unroll
                for (int u = 0; u < HB; ++u) acc[r] += h0 + u < a.Hkv ? v[r][u] : 0.f;
        }
#pragma unroll
        for (int r = 0; r < NREG; ++r) {
            const int j = r * nt + tid;
            if (j < V) {
                const float s = acc[r] * a.norm;
                key[j] = float_to_key(s);
                flag[j] = 0;
                if (a.scores_out) a.scores_out[(int64_t)b * a.V + j] = s;
            }
        }
    }
    if (a.meta)
        for (int i = keep + tid; i < a.keep; i += nt) a.kept_idx[(int64_t)b * a.keep + i] = -1;
    __syncthreads();
    auto slot = [&](int sl, int &idx) -> uint32_t {
        idx = sl;
        return key[sl];
    };
    if (GLOBAL_WAVE) {
        if (wave_id() == 0) wave_topk_regs<NREG>(slot, V, keep, flag, 1);
        __syncthreads();
    } else {
        block_topk_regs<NREG>(slot, V, keep, flag, 1, sm);
    }
    __syncthreads();  // the keys are no longer needed: their LDS holds the counts of the walk
    ranked_walk(flag, V, reinterpret_cast<int *>(key), [&](int j, bool kept, int s) {
        if (kept) a.kept_idx[(int64_t)b * a.keep + s] = j;
    });
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
static size_t round16(size_t v) { return (v + 15) & ~(size_t)15; }

size_t encoder_select_lds_bytes(int N, int has_local) {
    return sizeof(SelectSmem) + (size_t)N * 4 * (has_local ? 2 : 1) + round16((size_t)N);
}
size_t llm_select_lds_bytes(int V) { return sizeof(SelectSmem) + (size_t)V * 4 + round16((size_t)V); }

template <auto kernel, typename... Args>
static hipError_t launch_select(int blocks, int threads, size_t smem, hipStream_t s,
                                const Args &...args) {
    static std::atomic<uint64_t> lds_allowed{0};  // one per kernel instantiation
    if (smem > 64 * 1024) {
        hipError_t e = allow_large_lds(kernel, lds_allowed);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kernel, dim3(blocks), dim3(threads), smem, s, args...);
    return hipGetLastError();
}

hipError_t launch_encoder_select(const EncSelectArgs &a, hipStream_t s) {
    const int N = a.gh * a.gw, blocks = a.B * a.C;
    const size_t smem = encoder_select_lds_bytes(N, a.head_local != nullptr);
    // slots of the largest window: rows x columns padded to a power of two
    int wcols = 1;
    while (wcols < (a.gw + a.wc - 1) / a.wc) wcols <<= 1;
    const int win_slots = a.kw > 0 ? ((a.gh + a.wr - 1) / a.wr) * wcols : 0;
#define VSCAN_SEL(...) \
    return launch_select<encoder_select_kernel<__VA_ARGS__>>(blocks, threads, smem, s, a, 0)
    // WIN_MODE 3 keeps, behind the usual state, a window-major copy of the keys (pitch = slots of
    // the largest window, in whole 16-byte reads) and the two geometry tables
    const int win_pitch = ((((a.gh + a.wr - 1) / a.wr) * ((a.gw + a.wc - 1) / a.wc)) + 3) & ~3;
    const size_t smem_wm = round16(sizeof(SelectSmem) + (size_t)N * 4 * (a.head_local ? 2 : 1) + N) +
                           (size_t)a.wr * a.wc * win_pitch * 4 + (size_t)3 * (a.gh + a.gw) * 4;
#define VSCAN_SEL_WM(...)                                                                      \
    return launch_select<encoder_select_kernel<__VA_ARGS__>>(blocks, threads, smem_wm, s, a, \
                         win_pitch)
    if (N <= 1024) {
        // small segment: one thread per token, wave 0 does the global scan from registers
        int threads = (N + kWave - 1) / kWave * kWave;
        if (win_slots <= 128) {  // ranking by counting costs ~win_slots compares per token
            if (N <= 256) VSCAN_SEL_WM(3, 1, true, 4);
            if (N <= 640) VSCAN_SEL_WM(3, 1, true, 10);
            VSCAN_SEL_WM(3, 1, true, 16);
        }
        const int want = a.wr * a.wc * kWave;  // one wave per window where that fits
        if (want > threads) threads = want < 1024 ? want : 1024;
        if (win_slots <= 256) {
            if (N <= 640) VSCAN_SEL(1, 4, true, 10);
            VSCAN_SEL(1, 4, true, 16);
        }
        if (N <= 640) VSCAN_SEL(1, 32, true, 10);
        VSCAN_SEL(1, 32, true, 16);
    }
    const int threads = 1024;  // large segment: block-wide global scan, ceil(N/1024) registers
    const int nreg = (N + threads - 1) / threads;
    const int max_window = ((a.gh + a.wr - 1) / a.wr) * ((a.gw + a.wc - 1) / a.wc);
    if (N > 4096 && a.pre_key_ws && a.pre_flag_ws && (a.kw <= 0 || max_window <= 1024)) {
        // windows (and head sums) by a workgroup each, then the global scan by one per segment
        const int wthreads = a.kw > 0 ? (max_window + kWave - 1) / kWave * kWave : 1024;
        dim3 grid(a.kw > 0 ? a.wr * a.wc : (N + 1023) / 1024, blocks);
        hipLaunchKernelGGL(encoder_select_local_kernel, grid, dim3(wthreads), 0, s, a, a.pre_key_ws,
                           a.pre_flag_ws);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        EncSelectArgs g = a;
        g.pre_key = a.pre_key_ws;
        g.pre_flag = a.pre_flag_ws;
        g.scores_out = nullptr;  // written by the first kernel
        if (nreg <= 4) return launch_select<encoder_select_kernel<2, 1, false, 4>>(blocks, threads, smem, s, g, 0);
        if (nreg <= 16) return launch_select<encoder_select_kernel<2, 1, false, 16>>(blocks, threads, smem, s, g, 0);
        return launch_select<encoder_select_kernel<2, 1, false, 32>>(blocks, threads, smem, s, g, 0);
    }
    if (win_slots * nreg <= 128) {
        if (nreg <= 4) VSCAN_SEL(0, 1, false, 4);
        if (nreg <= 16) VSCAN_SEL(0, 1, false, 16);
        VSCAN_SEL(0, 1, false, 32);
    }
    if (win_slots <= 256) {
        if (nreg <= 4) VSCAN_SEL(1, 4, false, 4);
        if (nreg <= 16) VSCAN_SEL(1, 4, false, 16);
        VSCAN_SEL(1, 4, false, 32);
    }
    if (win_slots <= 2048) {
        if (nreg <= 4) VSCAN_SEL(1, 32, false, 4);
        if (nreg <= 16) VSCAN_SEL(1, 32, false, 16);
        VSCAN_SEL(1, 32, false, 32);
    }
    // one register count serves the window searches and the global one; a window padded to a
    // power of two may hold up to twice the segment's tokens
    const int nreg_w = (win_slots + threads - 1) / threads;
    const int nreg_both = nreg_w > nreg ? nreg_w : nreg;
    if (nreg_both <= 4) VSCAN_SEL(2, 1, false, 4);
    if (nreg_both <= 16) VSCAN_SEL(2, 1, false, 16);
    if (nreg_both <= 32) VSCAN_SEL(2, 1, false, 32);
    VSCAN_SEL(2, 1, false, 64);
#undef VSCAN_SEL
#undef VSCAN_SEL_WM
}

hipError_t launch_llm_select(const LlmSelectArgs &a, hipStream_t s) {
    const size_t smem = llm_select_lds_bytes(a.V);
    if (a.V <= 1024) {
        const int threads = (a.V + kWave - 1) / kWave * kWave;
        if (a.V <= 256)
            return launch_select<llm_select_kernel<true, 4>>(a.B, threads, smem, s, a);
        return launch_select<llm_select_kernel<true, 16>>(a.B, threads, smem, s, a);
    }
    const int nreg = (a.V + 1023) / 1024;
    if (nreg <= 4) return launch_select<llm_select_kernel<false, 4>>(a.B, 1024, smem, s, a);
    if (nreg <= 16) return launch_select<llm_select_kernel<false, 16>>(a.B, 1024, smem, s, a);
    return launch_select<llm_select_kernel<false, 32>>(a.B, 1024, smem, s, a);
}

}  // namespace vscan
