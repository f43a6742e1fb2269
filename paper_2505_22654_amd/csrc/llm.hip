// Stage 2 (Sec. 4.2): text-to-visual attention scoring (Eq. 5) and the
// order-preserving compaction of hidden states and K/V ("Remarks on KV Cache").
#include <algorithm>

#include "common.hpp"
#include "launch.hpp"

namespace vscan {

// ---------------------------------------------------------------------------
// Scoring.  An item is one (sequence, kv head): its keys are streamed once from
// HBM and multiplied on the matrix cores with all the query rows sharing the kv
// head (R = (Hq/Hkv) * Tq rows, padded to 16 per block).  Logits stay in LDS until
// the row maxima / sums are known, then the normalised rows are summed in a fixed
// order into
//   part[b][g][j] = sum_r softmax(row r)_j          (j over the visual span).
//
// How the keys reach the matrix cores (STAGED): a 16x16 operand wants lane l to
// hold 16 bytes of key (l % 16), so loading operands straight from memory makes
// every quarter-wave touch 16 different rows.  Instead a wave fetches a tile (16
// consecutive keys = 16 * row_bytes contiguous bytes) fully coalesced, 1 KiB per
// instruction, drops it into a private LDS staging area with padded rows and reads
// it back in operand layout.  Only this wave touches its staging area and the LDS
// operations of one wave complete in order, so no barrier is involved.  All global
// addresses are clamped into the key range (never predicated), which keeps the
// loads independent: the compiler waits only for the tile it is about to use while
// the later tiles stay in flight.  When the staging areas do not fit in
// LDS beside the logits, the operands are loaded directly (!STAGED).
//
// The logits of a long span leave LDS room for one workgroup per CU, so nothing
// else would keep that CU's memory pipe busy while the workgroup normalises.  The
// grid is therefore persistent (a workgroup takes items blockIdx.x, + gridDim.x,
// ...) and the tile stream runs across items: during the last round of an item the
// first tiles of the next item are already being fetched (and its queries right
// after), and they arrive while the softmax epilogue runs.
// ---------------------------------------------------------------------------
// DEPTH = 16-key tiles a wave keeps in flight: four for long spans, two for the widest rows
// (register budget) and for short spans, where a wave has no more than two tiles per item and
// the smaller register footprint lets a second workgroup share the CU.
constexpr int kScoreWaves = 8;  // waves per workgroup
constexpr int kScoreHeader = 128 + kScoreWaves * 64;  // floats of LDS before the logits

__host__ __device__ inline int score_logit_stride(int nk) {
    // floats per logit row: >= nk rounded up to 16, and = 16 mod 64 so that the 16 query rows
    // a wave writes at once start in different LDS banks
    const int nk16 = (nk + 15) & ~15;
    return nk16 + ((16 - nk16 % 64) + 64) % 64;
}

template <typename T, int NC, int NRB, bool STAGED, int DEPTH>
__global__ __launch_bounds__(kScoreWaves * kWave, (DEPTH == 2 && NC <= 4 && NRB == 1) ? 4 : 2) void llm_score_kernel(const T *__restrict__ q,
                                                        const T *__restrict__ k,
                                                        float *__restrict__ part, int B, int Hq,
                                                        int Hkv, int Tq, int S_cap, int dh,
                                                        int vis_start_u, int V_cap, int k0_u,
                                                        int nk_u, int domain_all,
                                                        const SeqMeta *__restrict__ meta,
                                                        float sl2) {
    // S_cap, V_cap: rows per sequence of k and of part (tensor strides).  Without `meta` every
    // sequence has the lengths (S_cap, vis_start_u, V_cap) and the key domain [k0_u, k0_u + nk_u);
    // with it, sequence b has those of meta[b], and nk_u is the longest domain (LDS layout).
    constexpr int STR = NC * 64 + 16;          // bytes per key in a staging area
    extern __shared__ __align__(16) unsigned char smem[];
    float *rowM = reinterpret_cast<float *>(smem);  // 64: row maxima
    float *rowInvL = rowM + 64;                      // 64: 1 / row sums
    float *waveM = rowInvL + 64;                     // [waves][64]: per-wave row maxima
    float *z = rowM + kScoreHeader;                  // [R][zs]

    const int group = Hq / Hkv, R = group * Tq;
    const int zs = score_logit_stride(nk_u);
    const int row_bytes = dh * (int)sizeof(T);
    const int lane = lane_id(), l16 = lane & 15, g = lane >> 4, w = wave_id();
    unsigned char *stage = reinterpret_cast<unsigned char *>(z + (int64_t)R * zs) + w * 16 * STR;
    const int items = B * Hkv;

    auto q_of = [&](int item) {  // item = b * Hkv + kv head; its query rows are contiguous
        return reinterpret_cast<const unsigned char *>(q) + (int64_t)item * group * Tq * row_bytes;
    };
    struct Geom {
        int S, vs, V, k0, nk;  // sequence length, visual span, key domain of an item
    };
    auto geom_of = [&](int item) {
        Geom gm = {S_cap, vis_start_u, V_cap, k0_u, nk_u};
        if (meta) {
            const SeqMeta m = meta[item / Hkv];
            gm.S = m.seq_len;
            gm.vs = m.vis_start;
            gm.V = m.vis_len;
            gm.k0 = domain_all ? 0 : m.vis_start;
            gm.nk = domain_all ? m.seq_len : m.vis_len;
        }
        return gm;
    };
    auto k_of = [&](int item, int k0) {
        return reinterpret_cast<const unsigned char *>(k) +
               ((int64_t)item * S_cap + k0) * row_bytes;
    };
    auto load_q = [&](const unsigned char *qbase, uint4(&dst)[NRB][NC]) {
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const int row = rb * 16 + l16;
                dst[rb][c] = load16_guard(qbase, (int64_t)row * row_bytes + 64 * c + 16 * g,
                                          row < R && 64 * c + 16 * g < row_bytes);
            }
    };

    // STAGED: piece m of a tile that this lane fetches is byte 1024 m + 16 lane of the tile's
    // 16 * row_bytes contiguous bytes.  tile_lds[m]: where it goes in the staging area (key
    // o / row_bytes, column o % row_bytes); a lane past the end of the tile drops what it
    // fetched into the padding of key 0, which nothing reads.
    int tile_lds[NC];
    if constexpr (STAGED) {
#pragma unroll
        for (int m = 0; m < NC; ++m) {
            const int o = 1024 * m + 16 * lane;
            const int r = o / row_bytes;
            tile_lds[m] = o < 16 * row_bytes ? r * STR + (o - r * row_bytes) : NC * 64;
        }
        // columns past the end of a key are never written again and must not hold NaN patterns
        for (int i = lane * 16; i < 16 * STR; i += kWave * 16)
            *reinterpret_cast<uint4 *>(stage + i) = zero16();
    }

    Geom gc;  // the item being multiplied; set at the top of every item
    uint4 ring[DEPTH][NC];
    // tile n of the item whose keys start at kbase and whose key domain is nk keys long
    auto fetch = [&](const unsigned char *kbase, int nk, int n, uint4(&dst)[NC]) {
        const int key0 = (w + kScoreWaves * n) * 16;
        if constexpr (STAGED) {
            // byte offsets are clamped to the last piece of the key range: always readable
            const int last_piece = nk * row_bytes - 16;
#pragma unroll
            for (int m = 0; m < NC; ++m)
                dst[m] = load16_stream(kbase,
                                       min(key0 * row_bytes + 1024 * m + 16 * lane, last_piece));
        } else {
            const int key = key0 + l16;
            const bool ok = key < nk;
#pragma unroll
            for (int c = 0; c < NC; ++c)
                dst[c] = load16_stream_guard(kbase, (int64_t)key * row_bytes + 64 * c + 16 * g,
                                             ok && 64 * c + 16 * g < row_bytes);
        }
    };

    uint4 qfrag[NRB][NC];
    float mx[NRB];  // running maximum of the logits this lane has filed, per row block
    // multiplies tile n (held in `tile`) with the query rows and files the logits
    auto process = [&](int n, const uint4(&tile)[NC]) {
        const int key0 = (w + kScoreWaves * n) * 16;
        uint4 kf[NC];  // operand layout: key l16, bytes 64 c + 16 g
        if constexpr (STAGED) {
#pragma unroll
            for (int m = 0; m < NC; ++m)
                *reinterpret_cast<uint4 *>(stage + tile_lds[m]) = tile[m];
#pragma unroll
            for (int c = 0; c < NC; ++c)
                kf[c] = *reinterpret_cast<const uint4 *>(stage + l16 * STR + 64 * c + 16 * g);
        } else {
#pragma unroll
            for (int c = 0; c < NC; ++c) kf[c] = tile[c];
        }
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
            f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < NC; ++c) mma16_chunk<T>(acc, kf[c], qfrag[rb][c]);
            // acc[r]: key key0 + 4g + r, query row rb*16 + l16
            const int row = rb * 16 + l16;
            if (row < R) {
                const int t = row % Tq;
                const int last_pos = gc.S - Tq + t;  // causal limit of this query
                float4 o;
                float *op = &o.x;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int kk = key0 + 4 * g + r;
                    op[r] = (kk < gc.nk && gc.k0 + kk <= last_pos) ? acc[r] * sl2 : -INFINITY;
                }
                mx[rb] = fmaxf(fmaxf(mx[rb], fmaxf(o.x, o.y)), fmaxf(o.z, o.w));
                *reinterpret_cast<float4 *>(z + (int64_t)row * zs + key0 + 4 * g) = o;
            }
        }
    };

    int item = blockIdx.x;
    if (item >= items) return;
    gc = geom_of(item);
    const unsigned char *kbase = k_of(item, gc.k0);
    load_q(q_of(item), qfrag);
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) fetch(kbase, gc.nk, d, ring[d]);

    for (; item < items; item += gridDim.x) {
        const bool has_next = item + (int)gridDim.x < items;
        const int next = has_next ? item + (int)gridDim.x : item;
        const Geom gn = has_next ? geom_of(next) : gc;
        const unsigned char *kbase_next = k_of(next, gn.k0);
        const int nk16 = (gc.nk + 15) & ~15, ntiles = nk16 >> 4;
        // this wave's tiles of the item: w, w + kScoreWaves, ...; every wave runs the same
        // number of rounds of DEPTH tiles, the surplus tiles are fetched (clamped) and ignored
        const int my_tiles = ntiles > w ? (ntiles - w + kScoreWaves - 1) / kScoreWaves : 0;
        const int rounds = ((ntiles + kScoreWaves - 1) / kScoreWaves + DEPTH - 1) / DEPTH;
        const int full_rounds = my_tiles / DEPTH;
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) mx[rb] = -INFINITY;

        // Round r works on tiles DEPTH r .. DEPTH r + DEPTH - 1 and refills each ring slot with
        // the tile of the next round - in the last round, with the first tiles of the next item.
        // Full rounds carry no condition, so each tile is awaited on its own while the later
        // ones stay in flight.
        int r = 0;
        if (full_rounds > 0 && rounds > 1) {
            // The first round is kept out of the loop below: here the stores of the previous
            // item's scores may still be pending next to the prefetched tiles, and the wait
            // that sorts that out should not be paid in every round.
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {
                process(d, ring[d]);
                fetch(kbase, gc.nk, DEPTH + d, ring[d]);
            }
            r = 1;
        }
        for (; r < full_rounds && r + 1 < rounds; ++r) {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {
                process(DEPTH * r + d, ring[d]);
                fetch(kbase, gc.nk, DEPTH * (r + 1) + d, ring[d]);
            }
        }
        for (; r < rounds; ++r) {  // the last round, and a partial one before it if there is one
            const bool last = r + 1 == rounds;
            const unsigned char *fbase = last ? kbase_next : kbase;
            const int fnk = last ? gn.nk : gc.nk;
            const int fn = last ? 0 : DEPTH * (r + 1);
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {
                if (DEPTH * r + d < my_tiles) process(DEPTH * r + d, ring[d]);
                if (!last || has_next) fetch(fbase, fnk, fn + d, ring[d]);
            }
        }
        if (has_next) load_q(q_of(next), qfrag);  // this item's queries are no longer needed

        // row maxima: over this lane's logits, the four key groups of the wave, the waves
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
            float m = mx[rb];
            m = fmaxf(m, __shfl_xor(m, 16, kWave));
            m = fmaxf(m, __shfl_xor(m, 32, kWave));
            if (g == 0) waveM[w * 64 + rb * 16 + l16] = m;
        }
        __syncthreads();

        // one wave per row: exponentials against the row maximum, written back over the
        // logits, and their sum
        for (int row = w; row < R; row += kScoreWaves) {
            float m = waveM[row];
#pragma unroll
            for (int ww = 1; ww < kScoreWaves; ++ww) m = fmaxf(m, waveM[ww * 64 + row]);
            float4 *zr = reinterpret_cast<float4 *>(z + (int64_t)row * zs);
            float sum = 0.f;
            for (int j = lane; j < (nk16 >> 2); j += kWave) {
                float4 v = zr[j];
                v.x = __builtin_amdgcn_exp2f(v.x - m);
                v.y = __builtin_amdgcn_exp2f(v.y - m);
                v.z = __builtin_amdgcn_exp2f(v.z - m);
                v.w = __builtin_amdgcn_exp2f(v.w - m);
                zr[j] = v;
                sum += (v.x + v.y) + (v.z + v.w);
            }
            sum = wave_sum(sum);
            if (lane == 0) rowInvL[row] = 1.0f / sum;
        }
        __syncthreads();

        // columns: sum over the rows in a fixed order
        float *out = part + (int64_t)item * V_cap;
        const int col0 = gc.vs - gc.k0;
        for (int j = threadIdx.x; j < gc.V; j += blockDim.x) {
            float s = 0.f;
            for (int row = 0; row < R; ++row) s += z[(int64_t)row * zs + col0 + j] * rowInvL[row];
            out[j] = s;
        }
        if (!has_next) break;
        __syncthreads();  // the logits are free for the next item

        kbase = kbase_next;
        gc = gn;
    }
}

// LDS bytes: header, logits, and (staged) one tile per wave
static size_t llm_score_lds(int rows, int nk, int nc, bool staged) {
    return (size_t)(kScoreHeader + (int64_t)rows * score_logit_stride(nk)) * sizeof(float) +
           (staged ? (size_t)kScoreWaves * 16 * (nc * 64 + 16) : 0);
}
constexpr size_t kScoreLdsMax = 160 * 1024;

bool llm_score_supported(int rows, int nk, int row_bytes) {
    return rows <= 64 && row_bytes <= 512 &&
           llm_score_lds(rows, nk, (row_bytes + 63) / 64, false) <= kScoreLdsMax;
}

template <typename T, int NC, int NRB, bool STAGED, int DEPTH>
static hipError_t llm_score_launch3(const LlmScoreArgs &a, hipStream_t s, size_t smem) {
    const int k0 = a.domain_all ? 0 : a.vis_start;
    const int nk = a.domain_all ? a.S : a.V;
    static std::atomic<uint64_t> lds_allowed{0};  // one per instantiation
    if (smem > 64 * 1024) {
        hipError_t e = allow_large_lds(llm_score_kernel<T, NC, NRB, STAGED, DEPTH>, lds_allowed);
        if (e != hipSuccess) return e;
    }
    // persistent grid: as many workgroups as the CUs hold at once (LDS decides, at most four
    // per CU), each taking every gridDim.x-th item
    const int64_t items = (int64_t)a.B * a.Hkv;
    const int per_cu = (int)std::min<size_t>(4, std::max<size_t>(1, kScoreLdsMax / smem));
    const int grid = (int)std::min<int64_t>(items, (int64_t)kCus * per_cu);
    hipLaunchKernelGGL((llm_score_kernel<T, NC, NRB, STAGED, DEPTH>), dim3(grid),
                       dim3(kScoreWaves * kWave), smem, s, (const T *)a.q, (const T *)a.k, a.part,
                       a.B, a.Hq, a.Hkv, a.Tq, a.S, a.dh, a.vis_start, a.V, k0, nk, a.domain_all,
                       a.meta, a.scale * 1.4426950408889634f);
    return hipGetLastError();
}

template <typename T, int NC, int NRB, bool STAGED>
static hipError_t llm_score_launch2(const LlmScoreArgs &a, hipStream_t s, size_t smem) {
    const int nk = a.domain_all ? a.S : a.V;
    const int tiles_per_wave = ((nk + 15) / 16 + kScoreWaves - 1) / kScoreWaves;
    if (NC >= 8 || tiles_per_wave <= 2) return llm_score_launch3<T, NC, NRB, STAGED, 2>(a, s, smem);
    return llm_score_launch3<T, NC, NRB, STAGED, 4>(a, s, smem);
}

template <typename T, int NC, int NRB>
static hipError_t llm_score_launch(const LlmScoreArgs &a, hipStream_t s) {
    const int rows = (a.Hq / a.Hkv) * a.Tq;
    const int nk = a.domain_all ? a.S : a.V;
    const size_t staged = llm_score_lds(rows, nk, NC, true);
    // (the widest rows with many query rows would spill registers in the staged form)
    if (staged <= kScoreLdsMax && !(NC >= 8 && NRB >= 4))
        return llm_score_launch2<T, NC, NRB, true>(a, s, staged);
    return llm_score_launch2<T, NC, NRB, false>(a, s, llm_score_lds(rows, nk, NC, false));
}

template <typename T>
static hipError_t llm_score_t(const LlmScoreArgs &a, hipStream_t s) {
    const int rows = (a.Hq / a.Hkv) * a.Tq;
    const int nc = (a.dh * (int)sizeof(T) + 63) / 64;
    if (rows <= 16) {
        if (nc <= 2) return llm_score_launch<T, 2, 1>(a, s);
        if (nc <= 4) return llm_score_launch<T, 4, 1>(a, s);
        return llm_score_launch<T, 8, 1>(a, s);
    }
    if (nc <= 2) return llm_score_launch<T, 2, 4>(a, s);
    if (nc <= 4) return llm_score_launch<T, 4, 4>(a, s);
    return llm_score_launch<T, 8, 4>(a, s);
}

// ---------------------------------------------------------------------------
// Few (sequence, kv head) items with long key domains: one workgroup per item would leave most
// of the chip idle (a 4096-token span under 4 kv heads: 4 workgroups on 256 CUs), so the key
// domain is cut into chunks of 256 keys, one workgroup each.
//   llm_score_split_kernel    thread = key: logits of all R query rows against it, then per
//                             chunk and row the maximum m_c[r], the sum l_c[r] of
//                             e = 2^(z - m_c[r]), and e itself for the visual columns
//   llm_score_combine_kernel  M_r = max_c m_c[r], L_r = sum_c l_c[r] 2^(m_c[r] - M_r) in chunk
//                             order, part[j] = sum_r e[r][j] 2^(m_c(j)[r] - M_r) / L_r in row
//                             order: fixed orders throughout, no atomics
// ---------------------------------------------------------------------------
constexpr int kSplitChunk = 64;   // keys per workgroup: four lanes share a key row

template <typename T, int RB>
__global__ __launch_bounds__(256) void llm_score_split_kernel(
    const T *__restrict__ q, const T *__restrict__ k, float *__restrict__ e_out,
    float *__restrict__ stats, int Hkv, int R, int Tq, int S, int dh, int vis_start, int V, int k0,
    int nk, float sl2) {
    constexpr int E = ElemTraits<T>::kPer16B;
    extern __shared__ __align__(16) unsigned char smem[];
    float *qs = reinterpret_cast<float *>(smem);   // [R][dh]
    float *red = qs + RB * dh;                      // [RB][4]: per-wave partial results
    const int item = blockIdx.y, chunk = blockIdx.x, nchunks = gridDim.x;
    const int tid = threadIdx.x;
    const T *qrow = q + (int64_t)item * R * dh;     // the item's query rows are contiguous
    for (int i = tid; i < R * dh; i += 256) qs[i] = load_elem<T>(qrow + i);
    for (int i = R * dh + tid; i < RB * dh; i += 256) qs[i] = 0.f;
    __syncthreads();

    // Four adjacent lanes share a key: lane `sub` takes the 16-byte pieces sub, sub + 4, ... of
    // its row (the four lanes read 64 contiguous bytes per request), so the serial chain of
    // multiply-adds per lane is a quarter of the row, and the chip sees four times the workgroups.
    const int sub = tid & 3;
    const int kk = chunk * kSplitChunk + (tid >> 2);  // key inside the domain
    const unsigned char *krow = reinterpret_cast<const unsigned char *>(
        k + ((int64_t)item * S + k0 + min(kk, nk - 1)) * dh);   // clamped: always readable
    float acc[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r) acc[r] = 0.f;
    const int npieces = dh / E;
    // eight pieces per lane at a time (a 256-element bf16 row in one round trip)
    constexpr int PB = 8;
    for (int p0 = 0; p0 < npieces; p0 += 4 * PB) {
        uint4 raw[PB];
#pragma unroll
        for (int u = 0; u < PB; ++u)
            raw[u] = load16_stream(krow, (int64_t)min(p0 + 4 * u + sub, npieces - 1) * 16);
#pragma unroll
        for (int u = 0; u < PB; ++u) {
            const int piece = p0 + 4 * u + sub;
            if (p0 + 4 * u < npieces) {  // uniform; a lane past the end of the row adds zeros
                float v[E];
                unpack16<T>(raw[u], v);
                const bool live = piece < npieces;
#pragma unroll
                for (int r = 0; r < RB; ++r) {
                    const float *qr = qs + r * dh + min(piece, npieces - 1) * E;
#pragma unroll
                    for (int e = 0; e < E; ++e) acc[r] = fmaf(live ? v[e] : 0.f, qr[e], acc[r]);
                }
            }
        }
    }
#pragma unroll
    for (int r = 0; r < RB; ++r) acc[r] = group_sum<4>(acc[r]);  // every lane of a key: its logit
    // masking: keys past the domain, and for a causal row the keys behind its query
    float z[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        const int last_pos = S - Tq + (r < R ? r % Tq : 0);
        z[r] = (r < R && kk < nk && k0 + kk <= last_pos) ? acc[r] * sl2 : -INFINITY;
    }
    // per row: maximum over the chunk, then e and its sum
    const int lane = lane_id(), w = wave_id();
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        const float m = wave_max(z[r]);
        if (lane == 0) red[r * 4 + w] = m;
    }
    __syncthreads();
    float mrow[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r)
        mrow[r] = fmaxf(fmaxf(red[r * 4], red[r * 4 + 1]), fmaxf(red[r * 4 + 2], red[r * 4 + 3]));
    __syncthreads();
    const int col = k0 + kk - vis_start;            // visual column of this key
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        const float e = mrow[r] > -INFINITY ? __builtin_amdgcn_exp2f(z[r] - mrow[r]) : 0.f;
        if (sub == 0 && r < R && kk < nk && col >= 0 && col < V)
            e_out[((int64_t)item * R + r) * V + col] = e;
        const float sum = wave_sum(sub == 0 ? e : 0.f);  // one lane per key counts
        if (lane == 0) red[r * 4 + w] = sum;
    }
    __syncthreads();
    if (tid < R) {
        float m = -INFINITY;  // mrow[tid] without indexing registers by a run-time value
#pragma unroll
        for (int r = 0; r < RB; ++r)
            if (r == tid) m = mrow[r];
        float *st = stats + (((int64_t)item * nchunks + chunk) * R + tid) * 2;
        st[0] = m;
        st[1] = (red[tid * 4] + red[tid * 4 + 1]) + (red[tid * 4 + 2] + red[tid * 4 + 3]);
    }
}

__global__ __launch_bounds__(256) void llm_score_combine_kernel(const float *__restrict__ e_in,
                                                               const float *__restrict__ stats,
                                                               float *__restrict__ part, int R,
                                                               int V, int vis_start, int k0,
                                                               int nchunks) {
    extern __shared__ float wgt[];                  // [nchunks][R], then M[R], invL[R], then the pairs
    float *M = wgt + nchunks * R, *invL = M + R, *st = invL + R;
    const int item = blockIdx.y, tid = threadIdx.x;
    // all (maximum, sum) pairs of the item into LDS at once: the row loops below would
    // otherwise be chains of dependent global loads
    for (int i = tid; i < nchunks * R * 2; i += 256) st[i] = stats[(int64_t)item * nchunks * R * 2 + i];
    __syncthreads();
    // per row: maximum and rescaled sum over the chunks, one wave per row, lanes over chunks
    // (a fixed reduction tree: the result does not depend on scheduling)
    for (int r = wave_id(); r < R; r += 4) {
        float m = -INFINITY;
        for (int c = lane_id(); c < nchunks; c += kWave) m = fmaxf(m, st[(c * R + r) * 2]);
        m = wave_max(m);
        float l = 0.f;
        for (int c = lane_id(); c < nchunks; c += kWave) {
            const float mc = st[(c * R + r) * 2];
            if (mc > -INFINITY) l += st[(c * R + r) * 2 + 1] * __builtin_amdgcn_exp2f(mc - m);
        }
        l = wave_sum(l);
        if (lane_id() == 0) {
            M[r] = m;
            invL[r] = 1.0f / l;
        }
    }
    __syncthreads();
    for (int i = tid; i < nchunks * R; i += 256) {
        const int r = i % R;
        const float mc = st[i * 2];
        wgt[i] = mc > -INFINITY ? __builtin_amdgcn_exp2f(mc - M[r]) * invL[r] : 0.f;
    }
    __syncthreads();
    const int col = blockIdx.x * 256 + tid;
    if (col >= V) return;
    const int c = (vis_start + col - k0) / kSplitChunk;
    float sum = 0.f;
    for (int r = 0; r < R; ++r) sum += e_in[((int64_t)item * R + r) * V + col] * wgt[c * R + r];
    part[(int64_t)item * V + col] = sum;
}

// chunks the key domain is cut into, 0 when the one-workgroup-per-item kernel is the better fit
int llm_score_split_chunks(int B, int Hkv, int rows, int nk, bool ragged) {
    if (ragged || rows > 16 || nk < 1024 || (int64_t)B * Hkv > kCus / 4) return 0;
    return (nk + kSplitChunk - 1) / kSplitChunk;
}

template <typename T>
static hipError_t llm_score_split_t(const LlmScoreArgs &a, hipStream_t s, int nchunks) {
    const int R = (a.Hq / a.Hkv) * a.Tq, items = a.B * a.Hkv;
    const int k0 = a.domain_all ? 0 : a.vis_start, nk = a.domain_all ? a.S : a.V;
    const float sl2 = a.scale * 1.4426950408889634f;
    dim3 grid(nchunks, items);
    if (R <= 8) {
        const size_t smem = (size_t)(8 * a.dh + 8 * 4) * sizeof(float);
        hipLaunchKernelGGL((llm_score_split_kernel<T, 8>), grid, dim3(256), smem, s, (const T *)a.q,
                           (const T *)a.k, a.split_e, a.split_stats, a.Hkv, R, a.Tq, a.S, a.dh,
                           a.vis_start, a.V, k0, nk, sl2);
    } else {
        const size_t smem = (size_t)(16 * a.dh + 16 * 4) * sizeof(float);
        hipLaunchKernelGGL((llm_score_split_kernel<T, 16>), grid, dim3(256), smem, s, (const T *)a.q,
                           (const T *)a.k, a.split_e, a.split_stats, a.Hkv, R, a.Tq, a.S, a.dh,
                           a.vis_start, a.V, k0, nk, sl2);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t smem2 = (size_t)(3 * nchunks * R + 2 * R) * sizeof(float);
    hipLaunchKernelGGL(llm_score_combine_kernel, dim3((a.V + 255) / 256, items), dim3(256), smem2, s,
                       (const float *)a.split_e, (const float *)a.split_stats, a.part, R, a.V,
                       a.vis_start, k0, nchunks);
    return hipGetLastError();
}

hipError_t launch_llm_score(const LlmScoreArgs &a, hipStream_t s) {
    const int rows = (a.Hq / a.Hkv) * a.Tq;
    const int nchunks = llm_score_split_chunks(a.B, a.Hkv, rows, a.domain_all ? a.S : a.V,
                                               a.meta != nullptr);
    if (nchunks > 0 && a.split_e && a.split_stats)
        return a.is_bf16 ? llm_score_split_t<bf16_t>(a, s, nchunks)
                         : llm_score_split_t<float>(a, s, nchunks);
    return a.is_bf16 ? llm_score_t<bf16_t>(a, s) : llm_score_t<float>(a, s);
}

// ---------------------------------------------------------------------------
// Compaction.  New row p of a sequence comes from old row
//   p                          p <  vis_start
//   vis_start + kept[p - vs]   p <  vis_start + keep
//   p + (V - keep)             otherwise
// so sources never lie below destinations.  A "strip" is up to 256 bytes of one
// row of one slab (K or V: one (sequence, kv head); hidden: one sequence).
// ---------------------------------------------------------------------------
struct Strip {
    unsigned char *src, *dst;  // first byte of row 0 of the strip
    int64_t src_stride, dst_stride;
    int width;                 // bytes, multiple of 16, <= 256
    int b;
};

// slab bases only: valid before the per-sequence lengths of a ragged batch are known
__device__ __forceinline__ Strip decode_strip(const CompactArgs &a, int id) {
    const int kv_w = a.dh * a.elem_bytes, hid_w = a.Dh * a.elem_bytes;
    const int kv_strips = (kv_w + 255) / 256, hid_strips = (hid_w + 255) / 256;
    const int n_kv = a.B * a.Hkv * kv_strips;
    Strip s;
    if (id < 2 * n_kv) {
        const bool is_v = id >= n_kv;
        const int r = is_v ? id - n_kv : id;
        const int slab = r / kv_strips, strip = r - slab * kv_strips;
        unsigned char *in = reinterpret_cast<unsigned char *>(is_v ? a.v : a.k);
        unsigned char *out = reinterpret_cast<unsigned char *>(is_v ? a.v_out : a.k_out);
        s.b = slab / a.Hkv;
        s.src_stride = kv_w;
        s.dst_stride = kv_w;
        s.src = in + (int64_t)slab * a.S * kv_w + strip * 256;
        s.dst = a.in_place ? s.src : out + (int64_t)slab * a.out_rows * kv_w + strip * 256;
        s.width = min(256, kv_w - strip * 256);
    } else {
        const int r = id - 2 * n_kv;
        const int b = r / hid_strips, strip = r - b * hid_strips;
        unsigned char *in = reinterpret_cast<unsigned char *>(a.hidden);
        unsigned char *out = reinterpret_cast<unsigned char *>(a.hidden_out);
        s.b = b;
        s.src_stride = hid_w;
        s.dst_stride = hid_w;
        s.src = in + (int64_t)b * a.S * hid_w + strip * 256;
        s.dst = a.in_place ? s.src : out + (int64_t)b * a.out_rows * hid_w + strip * 256;
        s.width = min(256, hid_w - strip * 256);
    }
    return s;
}

// Ragged batch: replace the lengths in the (by-value) argument block by those of sequence b.
// Returns the kept-index row of the sequence.
__device__ __forceinline__ const int32_t *sequence_view(CompactArgs &a, int b) {
    const int32_t *kept_b = a.kept_idx + (int64_t)b * a.keep;  // a.keep is still the stride here
    if (a.meta) {
        const SeqMeta m = a.meta[b];
        a.S = m.seq_len;
        a.vis_start = m.vis_start;
        a.V = m.vis_len;
        a.keep = m.keep;
    }
    return kept_b;
}

// Source rows of N output rows p[i].  The kept indices are fetched for every p from a clamped
// position (never predicated, and pinned ahead of the selects by an empty asm so the compiler
// cannot sink them into branches): the index loads of a tile are independent of each other and
// all in flight together; a value is used only inside the kept span.  With keep == 0 the
// table still holds one readable int.
template <int N>
__device__ __forceinline__ void src_rows(const CompactArgs &a, const int32_t *kept_b,
                                         const int *p, int *sr) {
    int kv[N];
#pragma unroll
    for (int i = 0; i < N; ++i)
        kv[i] = kept_b[min(max(p[i] - a.vis_start, 0), max(a.keep, 1) - 1)];
#pragma unroll
    for (int i = 0; i < N; ++i) asm volatile("" : "+v"(kv[i]));
#pragma unroll
    for (int i = 0; i < N; ++i) {
        // clamped: the index comes from device memory
        const int kept_row = a.vis_start + min(max(kv[i], 0), a.V - 1);
        sr[i] = p[i] < a.vis_start ? p[i]
                                   : (p[i] < a.vis_start + a.keep ? kept_row : p[i] + (a.V - a.keep));
    }
}

constexpr int kCompactRpt = 8;                   // rows per thread per tile
constexpr int kCompactTile = 16 * kCompactRpt;   // rows per tile (16 threads span a row)

// Makes the compiler wait (s_waitcnt vmcnt) until the loads that produced these
// registers have returned.  A workgroup barrier by itself does not wait for a
// thread's outstanding global loads, and the in-place walk must not let any thread
// store over a row another thread is still reading.
__device__ __forceinline__ void wait_for_loads(const uint4 *regs, int n) {
#pragma unroll
    for (int i = 0; i < n; ++i)
        asm volatile("" ::"v"(regs[i].x), "v"(regs[i].y), "v"(regs[i].z), "v"(regs[i].w));
}

// In place.  One workgroup walks one strip from the first row that moves to the
// end.  Per tile: every thread's loads have returned (wait_for_loads), barrier,
// then the stores.  Tiles are written in ascending order while the next tile's
// loads are already in flight, which is safe because a tile's stores end below
// every later tile's sources (source row >= destination row, both ascending).
__global__ __launch_bounds__(256) void compact_inplace_kernel(CompactArgs a) {
    __shared__ int red[4];
    const Strip s = decode_strip(a, blockIdx.x);
    const int32_t *kept_b = sequence_view(a, s.b);
    if (a.keep == a.V) return;  // nothing was pruned
    const int S_out = a.S - a.V + a.keep;
    const int tid = threadIdx.x;

    // first destination row whose source differs
    int first = a.keep;
    for (int i = tid; i < a.keep; i += blockDim.x)
        if (kept_b[i] != i) {
            first = i;
            break;
        }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) first = min(first, __shfl_xor(first, o, kWave));
    if (lane_id() == 0) red[wave_id()] = first;
    __syncthreads();
    first = min(min(red[0], red[1]), min(red[2], red[3]));
    const int p0 = a.vis_start + first;

    const int piece = tid & 15, rloc = tid >> 4;
    const bool col_ok = piece * 16 < s.width;
    auto load_tile = [&](int tile, uint4 *dst) {
        int pr[kCompactRpt], sr[kCompactRpt];  // all index fetches first, then all row fetches
#pragma unroll
        for (int i = 0; i < kCompactRpt; ++i) pr[i] = p0 + tile * kCompactTile + i * 16 + rloc;
        src_rows<kCompactRpt>(a, kept_b, pr, sr);
#pragma unroll
        for (int i = 0; i < kCompactRpt; ++i) {
            const int p = p0 + tile * kCompactTile + i * 16 + rloc;
            const bool ok = col_ok && p < S_out;
            dst[i] = load16_guard(s.src, (int64_t)sr[i] * s.src_stride + piece * 16, ok);
        }
    };
    auto store_tile = [&](int tile, const uint4 *v) {
#pragma unroll
        for (int i = 0; i < kCompactRpt; ++i) {
            const int p = p0 + tile * kCompactTile + i * 16 + rloc;
            if (col_ok && p < S_out)
                *reinterpret_cast<uint4 *>(s.dst + (int64_t)p * s.dst_stride + piece * 16) = v[i];
        }
    };
    const int ntiles = (S_out - p0 + kCompactTile - 1) / kCompactTile;
    if (ntiles <= 0) return;
    uint4 bufa[kCompactRpt], bufb[kCompactRpt];
    load_tile(0, bufa);
    for (int t = 0; t < ntiles; t += 2) {
        if (t + 1 < ntiles) load_tile(t + 1, bufb);
        wait_for_loads(bufa, kCompactRpt);
        __syncthreads();
        store_tile(t, bufa);
        if (t + 1 >= ntiles) break;
        if (t + 2 < ntiles) load_tile(t + 2, bufa);
        wait_for_loads(bufb, kCompactRpt);
        __syncthreads();
        store_tile(t + 1, bufb);
    }
}

// Out of place: a plain row gather; grid (strips, row tiles).
__global__ __launch_bounds__(256) void compact_gather_kernel(CompactArgs a) {
    const Strip s = decode_strip(a, blockIdx.x);
    const int32_t *kept_b = sequence_view(a, s.b);
    const int S_out = a.S - a.V + a.keep;
    const int piece = threadIdx.x & 15, rloc = threadIdx.x >> 4;
    if (piece * 16 >= s.width) return;
    uint4 v[kCompactRpt];
    int pr[kCompactRpt], sr[kCompactRpt];  // all index fetches first, then all row fetches
#pragma unroll
    for (int i = 0; i < kCompactRpt; ++i) pr[i] = blockIdx.y * kCompactTile + i * 16 + rloc;
    src_rows<kCompactRpt>(a, kept_b, pr, sr);
#pragma unroll
    for (int i = 0; i < kCompactRpt; ++i) {
        const int p = blockIdx.y * kCompactTile + i * 16 + rloc;
        const bool ok = p < S_out;
        v[i] = load16_guard(s.src, (int64_t)sr[i] * s.src_stride + piece * 16, ok);
    }
#pragma unroll
    for (int i = 0; i < kCompactRpt; ++i) {
        const int p = blockIdx.y * kCompactTile + i * 16 + rloc;
        if (p < S_out)
            *reinterpret_cast<uint4 *>(s.dst + (int64_t)p * s.dst_stride + piece * 16) = v[i];
    }
}

hipError_t launch_compact(const CompactArgs &a, hipStream_t s) {
    const int kv_strips = (a.dh * a.elem_bytes + 255) / 256;
    const int hid_strips = (a.Dh * a.elem_bytes + 255) / 256;
    const int strips = 2 * a.B * a.Hkv * kv_strips + a.B * hid_strips;
    if (a.in_place) {
        hipLaunchKernelGGL(compact_inplace_kernel, dim3(strips), dim3(256), 0, s, a);
    } else {
        dim3 grid(strips, (a.max_out_rows + kCompactTile - 1) / kCompactTile);
        hipLaunchKernelGGL(compact_gather_kernel, grid, dim3(256), 0, s, a);
    }
    return hipGetLastError();
}

}  // namespace vscan
