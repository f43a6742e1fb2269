// Attention scores computed from hidden states and the layer's projection weights, for a
// caller that has no Q and K yet: Eq. 5 as written (Q = x_last W_Q^h, K = x W_K^h; the queries
// are the last Tq positions of a sequence) and the [CLS] row of Eq. 1 (the query is row 0 of a
// segment).  The result is, per sequence, the sum over the query rows of their softmax weights
// on every visual token; selection and everything after it are the kernels of the Q/K form.
//
// The keys are never projected.  For one query row q of head h,
//     q . (W_K^h x_j) = (W_K^hT q) . x_j ,
// so the query is carried into hidden space once (qt = W_K^hT q, one vector of `hidden`
// entries per head and query position) and the logits are a single contraction of qt
// with the hidden states of the key domain: B*nk*hidden*Hq*Tq multiply-adds instead of the
// B*nk*hidden*Hkv*dh of a key projection (a factor dh*Hkv/(Hq*Tq), 128 for an MHA layer of
// head size 128 and one query position).
//
// Precision.  Inputs are bf16.  All three contractions run on the matrix cores with bf16
// operands and fp32 accumulation; q and qt are fp32 results that become operands again, so
// each is split into a sum of bf16 planes (value = hi + mid + lo, every plane the bf16
// rounding of what the previous ones left over: three planes carry 24 mantissa bits, i.e. the
// whole fp32 value) and the planes are contracted one after the other into the same
// accumulators.  The other operand (weights, hidden states) is bf16 already, so every product
// is exact and the only rounding is that of the fp32 accumulation.
//
// Steps (every contraction is C[p][s] = sum_k P[p][k] * S[s][k], both operands with the
// contraction axis contiguous; S is the large, streamed operand):
//   1. q   [B*Tq, Hq*dh]        P = the Tq query rows of every sequence,   S = W_Q rows
//   2. qt  [Hkv][B*g*Tq, Dh]    P = q planes of the group's heads,         S = W_K^T rows
//      (stored as bf16 planes straight from the accumulators)
//   3. l   [B][Hq*Tq, nk]       P = qt planes,                             S = hidden rows
//   4. softmax of every (sequence, query row), in place; 5. per key the sum over rows.
// Contractions with few output tiles split the contraction axis over `ksplit` workgroups;
// partial results are stored side by side and summed, in fixed order, by whichever kernel reads
// them next.
#include <algorithm>

#include "common.hpp"
#include "fused.hpp"
#include "launch.hpp"

namespace vscan {
namespace {

constexpr int kTargetWorkgroups = 512;        // two per compute unit before the axis is split

struct GemmDims {
    int rows_s, rows_p;   // valid rows of the two operands
    int k_bytes;          // contraction length in bytes (multiple of 16)
    int ksplit;
    int Z, s_tiles, p_tiles;  // batch entries and tiles per entry (set by the launcher)
    int affine;           // keep a batch entry's workgroups on one XCD (and its L2)
    float *c;             // [ksplit][Z][rows_p][rows_s]
};

// fp32 partial result of share ks
__device__ __forceinline__ void emit_partial(const GemmDims &d, int ks, int z, int p, int s_row,
                                             float v) {
    d.c[(((int64_t)ks * d.Z + z) * d.rows_p + p) * d.rows_s + s_row] = v;
}

// ---- operand addressing of the three contractions -------------------------------------------
// s_base/p_base: wave-uniform base of batch entry z (and plane pl); s_off/p_off: byte offset of a
// row's first contraction element from that base.

template <typename T>
struct ProbQ {
    using Elem = T;
    static constexpr int PL = 1;
    static constexpr bool kStreamS = false;
    GemmDims d;
    const char *hidden, *w_q;
    int Tq, S, q_row0, row_bytes;  // row_bytes = Dh * sizeof(T)
    const SeqMeta *meta;           // ragged batch: the queries are a sequence's own last rows
    __device__ int rows_s(int) const { return d.rows_s; }
    __device__ const char *s_base(int) const { return w_q; }
    __device__ uint32_t s_off(int n) const { return (uint32_t)n * (uint32_t)row_bytes; }
    __device__ const char *p_base(int, int) const { return hidden; }
    __device__ uint32_t p_off(int m) const {
        const int b = m / Tq, t = m - b * Tq;
        const int first = meta ? meta[b].seq_len - Tq : q_row0;
        return (uint32_t)(b * S + first + t) * (uint32_t)row_bytes;
    }
    __device__ void emit(int ks, int z, int p, int s_row, float v) const {
        emit_partial(d, ks, z, p, s_row, v);
    }
};

// q arrives as bf16 planes (bf16 inputs: three planes carry all 24 bits of the fp32 value) or as
// the fp32 values themselves (fp32 inputs: one "plane"); the result leaves the same way.
template <typename T>
struct ProbQt {
    using Elem = T;
    static constexpr int ES = (int)sizeof(T);
    static constexpr int PL = ES == 2 ? 3 : 1;
    static constexpr bool kStreamS = false;
    GemmDims d;
    const char *q_planes, *w_k_t;
    int Tq, group, dh, Hq, Hkv;
    int64_t plane_bytes;  // B*Tq*Hq*dh*ES
    __device__ int rows_s(int) const { return d.rows_s; }
    __device__ const char *s_base(int g) const { return w_k_t + (int64_t)g * dh * ES; }
    __device__ uint32_t s_off(int c) const { return (uint32_t)c * (uint32_t)(Hkv * dh * ES); }
    __device__ const char *p_base(int g, int pl) const {
        return q_planes + pl * plane_bytes + (int64_t)g * group * dh * ES;
    }
    __device__ uint32_t p_off(int m) const {  // m = (b*group + hh)*Tq + t
        const int t = m % Tq, bh = m / Tq;
        const int hh = bh % group, b = bh / group;
        return (uint32_t)((b * Tq + t) * Hq * dh + hh * dh) * (uint32_t)ES;
    }
    // the result goes out in its final form right away (this contraction is never split)
    uint16_t *qt_planes;      // bf16: [kFusedQtPlanes][Hkv][rows_p][rows_s]; fp32: [Hkv][rows_p][rows_s] floats
    int64_t qt_plane_elems;   // Hkv*rows_p*rows_s
    __device__ void emit(int, int g, int p, int s_row, float v) const {
        const int64_t at = ((int64_t)g * d.rows_p + p) * d.rows_s + s_row;
        if constexpr (ES == 4) {
            reinterpret_cast<float *>(qt_planes)[at] = v;
        } else {
            uint16_t *o = qt_planes + at;
#pragma unroll
            for (int pl = 0; pl < kFusedQtPlanes; ++pl) {
                const uint32_t bits = f32_to_bf16_rne(v);
                o[pl * qt_plane_elems] = (uint16_t)bits;
                v -= __uint_as_float(bits << 16);
            }
        }
    }
};

template <typename T, bool STREAM>
struct ProbLogit {
    using Elem = T;
    static constexpr int PL = sizeof(T) == 2 ? kFusedQtPlanes : 1;
    static constexpr bool kStreamS = STREAM;
    GemmDims d;
    const char *hidden, *qt_planes;
    int Tq, group, S, k0, row_bytes, Mg;  // Mg = B*group*Tq rows of qt per kv head
    int64_t plane_bytes;                  // Hkv*Mg*Dh*sizeof(T)
    const SeqMeta *meta;                  // ragged batch: key domain of sequence b from meta[b]
    int domain_all;
    __device__ int rows_s(int b) const {
        return meta ? (domain_all ? meta[b].seq_len : meta[b].vis_len) : d.rows_s;
    }
    __device__ const char *s_base(int b) const {
        const int first = meta ? (domain_all ? 0 : meta[b].vis_start) : k0;
        return hidden + ((int64_t)b * S + first) * row_bytes;
    }
    __device__ uint32_t s_off(int j) const { return (uint32_t)j * (uint32_t)row_bytes; }
    __device__ const char *p_base(int b, int pl) const {
        return qt_planes + pl * plane_bytes + (int64_t)b * group * Tq * row_bytes;
    }
    __device__ uint32_t p_off(int r) const {  // r = h*Tq + t
        const int t = r % Tq, h = r / Tq;
        const int g = h / group, hh = h - g * group;
        return (uint32_t)(g * Mg + hh * Tq + t) * (uint32_t)row_bytes;
    }
    __device__ void emit(int ks, int z, int p, int s_row, float v) const {
        emit_partial(d, ks, z, p, s_row, v);
    }
};

// Projection of every row of `hidden` with a weight matrix whose rows are output features; the
// result goes out in fp32 as [bc][head][token][e] (never split along the contraction axis).
template <typename T>
struct ProbProject {
    using Elem = T;
    static constexpr int PL = 1;
    static constexpr bool kStreamS = false;
    GemmDims d;
    const char *hidden, *w;
    int S, H, dh, row_bytes;
    float *out;
    __device__ int rows_s(int) const { return d.rows_s; }
    __device__ const char *s_base(int) const { return w; }
    __device__ uint32_t s_off(int n) const { return (uint32_t)n * (uint32_t)row_bytes; }
    __device__ const char *p_base(int, int) const { return hidden; }
    __device__ uint32_t p_off(int m) const { return (uint32_t)m * (uint32_t)row_bytes; }
    __device__ void emit(int, int, int p, int s_row, float v) const {
        const int bc = p / S, t = p - bc * S;
        const int h = s_row / dh, e = s_row - h * dh;
        out[(((int64_t)bc * H + h) * S + t) * dh + e] = v;
    }
};

// One workgroup of WS x WP waves: 32*FS*WS streamed rows x 32*FP*WP plane-operand rows, one
// share of the contraction axis; a wave owns FS x FP tiles of 32 x 32.  Both operands pass
// through LDS in CH-byte row chunks: the next chunk is fetched into registers (coalesced,
// CH/16 lanes per row) while the matrix cores work on the current one.  Row indices past the
// operand's end are clamped (the rows are computed and not stored); chunk pieces past the
// contraction length are fetched from a clamped offset and zeroed on their way into LDS.
template <class Prob, int WS, int WP, int FS, int FP, int CH>
__global__ __launch_bounds__(64 * WS * WP) void nt_gemm_kernel(Prob pr) {
    constexpr int kChunkBytes = CH, kRowPitch = CH + 16, PIECES = CH / 16;
    constexpr int PL = Prob::PL;
    constexpr int THREADS = 64 * WS * WP;
    constexpr int TS = 32 * FS * WS, TP = 32 * FP * WP;
    constexpr int ROWS_PER_PASS = THREADS / PIECES;      // rows one staging pass covers
    constexpr int NS = TS / ROWS_PER_PASS, NP = TP / ROWS_PER_PASS;
    static_assert(TS % ROWS_PER_PASS == 0 && TP % ROWS_PER_PASS == 0, "staging covers whole tiles");
    __shared__ __attribute__((aligned(16))) unsigned char lds_s[TS * kRowPitch];
    __shared__ __attribute__((aligned(16))) unsigned char lds_p[PL * TP * kRowPitch];

    const GemmDims d = pr.d;
    const int tid = threadIdx.x, lane = lane_id();
    const int ws = wave_id() % WS, wp = wave_id() / WS;
    int z, item;
    if (!image_affine_decode(d.Z, d.s_tiles * d.p_tiles * d.ksplit, d.affine != 0, z, item)) return;
    const int s_tile = item % d.s_tiles, rest = item / d.s_tiles;
    const int ptile = rest / d.ksplit, ks = rest - ptile * d.ksplit;
    const int s0 = s_tile * TS, p0 = ptile * TP;
    const int rows_s = pr.rows_s(z);  // this batch entry's own count (d.rows_s is the capacity)
    if (s0 >= rows_s) return;         // the whole workgroup: nothing of this tile exists
    const int nchunks = (d.k_bytes + kChunkBytes - 1) / kChunkBytes;
    const int cps = (nchunks + d.ksplit - 1) / d.ksplit;
    const int c_begin = ks * cps, c_end = min(nchunks, c_begin + cps);

    const int piece = tid % PIECES, srow = tid / PIECES;
    const char *sb = pr.s_base(z);
    const char *pb[PL];
#pragma unroll
    for (int pl = 0; pl < PL; ++pl) pb[pl] = pr.p_base(z, pl);
    uint32_t s_off[NS], p_off[NP];
#pragma unroll
    for (int i = 0; i < NS; ++i)
        s_off[i] = pr.s_off(min(s0 + srow + ROWS_PER_PASS * i, rows_s - 1));
#pragma unroll
    for (int i = 0; i < NP; ++i)
        p_off[i] = pr.p_off(min(p0 + srow + ROWS_PER_PASS * i, d.rows_p - 1));

    f32x16_t acc[FP][FS];
#pragma unroll
    for (int i = 0; i < FP; ++i)
#pragma unroll
        for (int j = 0; j < FS; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    uint4 rs[NS], rp[PL * NP];
    auto fetch = [&](int c) {
        const uint32_t col = (uint32_t)min(c * kChunkBytes + piece * 16, d.k_bytes - 16);
#pragma unroll
        for (int i = 0; i < NS; ++i)
            rs[i] = Prob::kStreamS ? load16_stream(sb, (int64_t)s_off[i] + col)
                                   : load16(sb, (int64_t)s_off[i] + col);
#pragma unroll
        for (int pl = 0; pl < PL; ++pl)
#pragma unroll
            for (int i = 0; i < NP; ++i) rp[pl * NP + i] = load16(pb[pl], (int64_t)p_off[i] + col);
    };

    // Workgroups walk their share of the contraction axis from staggered starting points (and
    // wrap around), so that at any moment the chip reads many different column ranges of the
    // row-strided operand rather than one (measured: a quarter faster on a cold pass over
    // 0.7 GB of hidden states).  The order depends on the grid position only.
    const int span = c_end - c_begin;
    // With many plane rows the workgroups of one batch entry keep a common order: they share
    // the plane operand's current chunk through L2.
    const unsigned start = (unsigned)z * 3u + (TP <= 64 ? (unsigned)s_tile * 5u : 0u);
    const int rot = span > 0 ? (int)(start % (unsigned)span) : 0;
    auto chunk_at = [&](int i) { const int r = i + rot; return c_begin + (r >= span ? r - span : r); };
    if (span > 0) fetch(chunk_at(0));
    for (int i = 0; i < span; ++i) {
        const int c = chunk_at(i);
        const bool valid = c * kChunkBytes + piece * 16 < d.k_bytes;
#pragma unroll
        for (int i = 0; i < NS; ++i)
            *reinterpret_cast<uint4 *>(lds_s + (srow + ROWS_PER_PASS * i) * kRowPitch + piece * 16) =
                valid ? rs[i] : zero16();
#pragma unroll
        for (int pl = 0; pl < PL; ++pl)
#pragma unroll
            for (int i = 0; i < NP; ++i)
                *reinterpret_cast<uint4 *>(lds_p + (pl * TP + srow + ROWS_PER_PASS * i) * kRowPitch +
                                           piece * 16) = valid ? rp[pl * NP + i] : zero16();
        __syncthreads();
        fetch(chunk_at(min(i + 1, span - 1)));  // unconditional; the last round re-reads its chunk
#pragma unroll
        for (int sub = 0; sub < kChunkBytes / 32; ++sub) {
            const int colb = sub * 32 + 16 * (lane >> 5);
            uint4 b[FS];
#pragma unroll
            for (int j = 0; j < FS; ++j)
                b[j] = *reinterpret_cast<const uint4 *>(
                    lds_s + ((ws * FS + j) * 32 + (lane & 31)) * kRowPitch + colb);
#pragma unroll
            for (int i = 0; i < FP; ++i)
#pragma unroll
                for (int pl = 0; pl < PL; ++pl) {
                    const uint4 a = *reinterpret_cast<const uint4 *>(
                        lds_p + (pl * TP + (wp * FP + i) * 32 + (lane & 31)) * kRowPitch + colb);
#pragma unroll
                    for (int j = 0; j < FS; ++j) mma32_chunk<typename Prob::Elem>(acc[i][j], a, b[j]);
                }
        }
        __syncthreads();
    }

    // acc[i][j][r] = C[p0 + 32 (wp FP + i) + acc_row(r)][s0 + 32 (ws FS + j) + lane % 32]: lanes
    // run along the streamed rows, which are contiguous in the result
#pragma unroll
    for (int j = 0; j < FS; ++j) {
        const int s_out = s0 + (ws * FS + j) * 32 + (lane & 31);
        if (s_out >= rows_s) continue;
#pragma unroll
        for (int i = 0; i < FP; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int p_out = p0 + (wp * FP + i) * 32 + acc_row(r);
                if (p_out < d.rows_p) pr.emit(ks, z, p_out, s_out, acc[i][j][r]);
            }
    }
}

// Tile shapes by the number of plane-operand rows: <= 32, <= 64, <= 128, more.  `ch` is the
// number of contraction bytes staged per step: the LDS row pitch is ch + 16 bytes (36 or 68
// words, so the 16-byte reads of eight consecutive rows fall into distinct banks).  With few
// plane rows the kernel streams the other operand from HBM, and longer contiguous pieces of
// its rows serve that better.
struct TileShape {
    int ts, tp, ch;
};
TileShape tile_shape(int rows_p, int rows_s, int Z) {
    if (rows_p <= 64) {
        // few plane rows: 256 streamed rows per workgroup when that still leaves a workgroup or
        // two per compute unit, else 128 (twice the workgroups, each with half the rows in flight)
        const int tp = rows_p <= 32 ? 32 : 64;
        const int64_t tiles = (int64_t)((rows_s + 255) / 256) * Z;
        return {tiles >= kTargetWorkgroups ? 256 : 128, tp, 128};
    }
    if (rows_p <= 128) return {256, 128, 128};
    return {256, 256, 128};
}

template <class Prob>
hipError_t launch_gemm(Prob pr, int Z, hipStream_t s) {
    GemmDims &d = pr.d;
    const TileShape t = tile_shape(d.rows_p, d.rows_s, Z);
    d.Z = Z;
    d.s_tiles = (d.rows_s + t.ts - 1) / t.ts;
    d.p_tiles = (d.rows_p + t.tp - 1) / t.tp;
    // with at least one batch entry per XCD, an entry's workgroups share the plane operand
    // through that XCD's L2
    d.affine = Z >= kXcds;
    const dim3 grid(image_affine_grid(Z, d.s_tiles * d.p_tiles * d.ksplit, d.affine != 0));
#define VSCAN_GEMM(WS, WP, FS, FP, CH) \
    hipLaunchKernelGGL((nt_gemm_kernel<Prob, WS, WP, FS, FP, CH>), grid, dim3(64 * WS * WP), 0, s, pr)
    if (t.tp == 32 && t.ts == 128)
        VSCAN_GEMM(4, 1, 1, 1, 128);
    else if (t.tp == 32)
        VSCAN_GEMM(4, 1, 2, 1, 128);
    else if (t.tp == 64 && t.ts == 128)
        VSCAN_GEMM(4, 1, 1, 2, 128);
    else if (t.tp == 64)
        VSCAN_GEMM(4, 1, 2, 2, 128);
    else if (t.tp == 128)
        VSCAN_GEMM(2, 2, 4, 2, 128);
    else
        VSCAN_GEMM(2, 4, 4, 2, 128);
#undef VSCAN_GEMM
    return hipGetLastError();
}

// value = sum of PL bf16 planes: plane p is the bf16 rounding of what planes < p left over
// (the remainders are exact in fp32).  Input: `ksplit` partial sums per element.
template <int PL>
__global__ __launch_bounds__(256) void split_planes_kernel(const float *__restrict__ c, int ksplit,
                                                           int64_t n, uint16_t *__restrict__ planes) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    float v = 0.f;
    for (int ks = 0; ks < ksplit; ++ks) v += c[ks * n + i];
#pragma unroll
    for (int pl = 0; pl < PL; ++pl) {
        const uint32_t bits = f32_to_bf16_rne(v);
        planes[pl * n + i] = (uint16_t)bits;
        v -= __uint_as_float(bits << 16);
    }
}

// Softmax of one (sequence, query row) over the key domain.  The scaled logits of the row
// (partial sums added in fixed order) stay in registers between the maximum, the sum of
// exponentials and the normalised weights, which overwrite the row's first partial slot.
// NREG * THREADS >= nk.  With `causal`, query position t of the Tq positions of a row index
// r = h*Tq + t sees all but the last Tq-1-t keys of the domain; the others get weight zero.
__device__ __forceinline__ int row_keys(int r, int nk, int Tq, int causal) {
    return causal ? nk - (Tq - 1 - r % Tq) : nk;
}
// Keys in the domain of sequence b: from the table of a ragged batch, else the common count.
// (With `causal` the domain is the whole sequence.)
__device__ __forceinline__ int domain_keys(const SeqMeta *meta, int b, int causal, int nk) {
    return meta ? (causal ? meta[b].seq_len : meta[b].vis_len) : nk;
}

template <int THREADS, int NREG>
__global__ __launch_bounds__(THREADS) void fused_softmax_kernel(float *__restrict__ c, int ksplit,
                                                                int64_t ks_stride, int nk_cap,
                                                                float scale, int Tq, int causal,
                                                                const SeqMeta *meta) {
    __shared__ float red[16];
    const int64_t row = (int64_t)blockIdx.y * gridDim.x + blockIdx.x;
    float *l = c + row * nk_cap;
    const int tid = threadIdx.x;
    const int nk = domain_keys(meta, blockIdx.y, causal, nk_cap);
    const int nv = row_keys(blockIdx.x, nk, Tq, causal);
    float v[NREG];
#pragma unroll
    for (int i = 0; i < NREG; ++i) v[i] = 0.f;
    for (int ks = 0; ks < ksplit; ++ks)
#pragma unroll
        for (int i = 0; i < NREG; ++i) v[i] += l[ks * ks_stride + min(tid + THREADS * i, nk - 1)];
    float m = -INFINITY;
#pragma unroll
    for (int i = 0; i < NREG; ++i) {
        v[i] *= scale;
        if (tid + THREADS * i < nv) m = fmaxf(m, v[i]);
    }
    m = block_max(m, red);
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < NREG; ++i) {
        v[i] = tid + THREADS * i < nv ? __expf(v[i] - m) : 0.f;
        sum += v[i];
    }
    sum = block_sum(sum, red);
    const float inv = 1.0f / sum;
#pragma unroll
    for (int i = 0; i < NREG; ++i)
        if (tid + THREADS * i < nk) l[tid + THREADS * i] = v[i] * inv;
}

// Rows too long for the register form: three passes over the row.
__global__ __launch_bounds__(1024) void fused_softmax_long_kernel(float *__restrict__ c, int ksplit,
                                                                  int64_t ks_stride, int nk_cap,
                                                                  float scale, int Tq, int causal,
                                                                  const SeqMeta *meta) {
    __shared__ float red[16];
    const int64_t row = (int64_t)blockIdx.y * gridDim.x + blockIdx.x;
    float *l = c + row * nk_cap;
    const int nk = domain_keys(meta, blockIdx.y, causal, nk_cap);
    const int nv = row_keys(blockIdx.x, nk, Tq, causal);
    float m = -INFINITY;
    for (int j = threadIdx.x; j < nv; j += 1024) {
        float v = 0.f;
        for (int ks = 0; ks < ksplit; ++ks) v += l[ks * ks_stride + j];
        v *= scale;
        l[j] = v;  // only this thread reads element j again
        m = fmaxf(m, v);
    }
    m = block_max(m, red);
    float sum = 0.f;
    for (int j = threadIdx.x; j < nv; j += 1024) sum += __expf(l[j] - m);
    sum = block_sum(sum, red);
    const float inv = 1.0f / sum;
    for (int j = threadIdx.x; j < nk; j += 1024) l[j] = j < nv ? __expf(l[j] - m) * inv : 0.f;
}

// part[b][j] = sum over the query rows of the softmax weight of visual token j (Eq. 5 before
// the division by the number of rows).  A workgroup owns 64 keys; its four waves take every
// fourth row and their sums are added in wave order.
__global__ __launch_bounds__(256) void fused_colsum_kernel(const float *__restrict__ p, int R,
                                                           int nk_cap, int vis_off, int V_cap,
                                                           int causal, const SeqMeta *meta,
                                                           float *__restrict__ part) {
    __shared__ float red[4][64];
    const int b = blockIdx.y;
    const int nk = domain_keys(meta, b, causal, nk_cap);
    int V = V_cap;
    if (meta) {
        V = meta[b].vis_len;
        vis_off = causal ? meta[b].vis_start : 0;
    }
    const int j = blockIdx.x * 64 + lane_id();
    const float *col = p + (int64_t)b * R * nk_cap + min(j, nk - 1);
    float acc = 0.f;
    int r = wave_id();
    for (; r + 28 < R; r += 32) {
        float t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = col[(int64_t)(r + 4 * u) * nk_cap];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += t[u];
    }
    for (; r < R; r += 4) acc += col[(int64_t)r * nk_cap];
    red[wave_id()][lane_id()] = acc;
    __syncthreads();
    const int t = j - vis_off;
    if (wave_id() == 0 && j < nk && t >= 0 && t < V)
        part[(int64_t)b * V_cap + t] =
            ((red[0][lane_id()] + red[1][lane_id()]) + red[2][lane_id()]) + red[3][lane_id()];
}

GemmDims dims(int rows_s, int rows_p, int k_elems, int es, int ksplit, float *c) {
    GemmDims d;
    d.rows_s = rows_s;
    d.rows_p = rows_p;
    d.k_bytes = k_elems * es;
    d.ksplit = ksplit;
    d.Z = d.s_tiles = d.p_tiles = 1;
    d.affine = 0;
    d.c = c;
    return d;
}

}  // namespace

int fused_ksplit(int rows_s, int rows_p, int Z, int k_elems, int elem_bytes) {
    const TileShape t = tile_shape(rows_p, rows_s, Z);
    const int64_t tiles = std::max<int64_t>(
        1, (int64_t)((rows_s + t.ts - 1) / t.ts) * ((rows_p + t.tp - 1) / t.tp) * Z);  // empty batch: 1
    const int nchunks = (k_elems * elem_bytes + t.ch - 1) / t.ch;
    int ks = (int)((kTargetWorkgroups + tiles - 1) / tiles);
    ks = max(1, min(ks, min(16, nchunks / 2)));
    return ks;
}

template <typename T>
static hipError_t fused_q_t(const FusedArgs &a, hipStream_t s) {
    ProbQ<T> pr;
    pr.d = dims(a.Hq * a.dh, a.B * a.Tq, a.Dh, (int)sizeof(T), a.ks_q, a.c_q);
    pr.hidden = reinterpret_cast<const char *>(a.hidden);
    pr.w_q = reinterpret_cast<const char *>(a.w_q);
    pr.Tq = a.Tq;
    pr.S = a.S;
    pr.q_row0 = a.q_row0;
    pr.meta = a.meta;
    pr.row_bytes = a.Dh * (int)sizeof(T);
    return launch_gemm(pr, 1, s);
}
hipError_t launch_fused_q(const FusedArgs &a, hipStream_t s) {
    return a.is_bf16 ? fused_q_t<bf16_t>(a, s) : fused_q_t<float>(a, s);
}

// fp32 inputs: q stays in fp32; the partial sums of the split contraction axis are added in
// fixed order
__global__ __launch_bounds__(256) void sum_partials_kernel(const float *__restrict__ c, int ksplit,
                                                           int64_t n, float *__restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    float v = 0.f;
    for (int ks = 0; ks < ksplit; ++ks) v += c[ks * n + i];
    out[i] = v;
}

hipError_t launch_fused_split_q(const FusedArgs &a, hipStream_t s) {
    const int64_t n = (int64_t)a.B * a.Tq * a.Hq * a.dh;
    if (a.is_bf16)
        hipLaunchKernelGGL(split_planes_kernel<3>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                           a.c_q, a.ks_q, n, a.q_planes);
    else
        hipLaunchKernelGGL(sum_partials_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                           a.c_q, a.ks_q, n, reinterpret_cast<float *>(a.q_planes));
    return hipGetLastError();
}

template <typename T>
static hipError_t fused_qt_t(const FusedArgs &a, hipStream_t s) {
    const int group = a.Hq / a.Hkv;
    ProbQt<T> pr;
    pr.d = dims(a.Dh, a.B * group * a.Tq, a.dh, (int)sizeof(T), 1, nullptr);
    pr.q_planes = reinterpret_cast<const char *>(a.q_planes);
    pr.w_k_t = reinterpret_cast<const char *>(a.w_k_t);
    pr.Tq = a.Tq;
    pr.group = group;
    pr.dh = a.dh;
    pr.Hq = a.Hq;
    pr.Hkv = a.Hkv;
    pr.plane_bytes = (int64_t)a.B * a.Tq * a.Hq * a.dh * (int64_t)sizeof(T);
    pr.qt_planes = a.qt_planes;
    pr.qt_plane_elems = (int64_t)a.B * a.Hq * a.Tq * a.Dh;
    return launch_gemm(pr, a.Hkv, s);
}
hipError_t launch_fused_qt(const FusedArgs &a, hipStream_t s) {
    return a.is_bf16 ? fused_qt_t<bf16_t>(a, s) : fused_qt_t<float>(a, s);
}

// Hidden states beyond this size cannot stay in the last-level cache between this pass and
// the compaction that follows; they are then fetched with the streaming hint, which a cold
// one-pass read is faster with.  Smaller ones keep plain loads, so the compaction finds them
// cached.
constexpr int64_t kStreamHiddenBytes = (int64_t)128 << 20;

template <typename T, bool STREAM>
hipError_t launch_logits(const FusedArgs &a, hipStream_t s) {
    const int group = a.Hq / a.Hkv;
    ProbLogit<T, STREAM> pr;
    pr.d = dims(a.nk, a.Hq * a.Tq, a.Dh, (int)sizeof(T), a.ks_l, a.c_l);
    pr.hidden = reinterpret_cast<const char *>(a.hidden);
    pr.qt_planes = reinterpret_cast<const char *>(a.qt_planes);
    pr.Tq = a.Tq;
    pr.group = group;
    pr.S = a.S;
    pr.k0 = a.k0;
    pr.row_bytes = a.Dh * (int)sizeof(T);
    pr.Mg = a.B * group * a.Tq;
    pr.plane_bytes = (int64_t)a.Hkv * pr.Mg * a.Dh * (int64_t)sizeof(T);
    pr.meta = a.meta;
    pr.domain_all = a.causal;
    return launch_gemm(pr, a.B, s);
}

hipError_t launch_fused_logits(const FusedArgs &a, hipStream_t s) {
    const bool stream = (int64_t)a.B * a.S * a.Dh * (a.is_bf16 ? 2 : 4) > kStreamHiddenBytes;
    if (a.is_bf16) return stream ? launch_logits<bf16_t, true>(a, s) : launch_logits<bf16_t, false>(a, s);
    return stream ? launch_logits<float, true>(a, s) : launch_logits<float, false>(a, s);
}

hipError_t launch_fused_softmax(const FusedArgs &a, hipStream_t s) {
    const int R = a.Hq * a.Tq;
    const int64_t ks_stride = (int64_t)a.B * R * a.nk;
    const dim3 grid(R, a.B);
#define VSCAN_SOFTMAX(T, N)                                                                      \
    hipLaunchKernelGGL((fused_softmax_kernel<T, N>), grid, dim3(T), 0, s, a.c_l, a.ks_l, ks_stride, \
                       a.nk, a.scale, a.Tq, a.causal, a.meta)
    if (a.nk <= 256)
        VSCAN_SOFTMAX(256, 1);
    else if (a.nk <= 1024)
        VSCAN_SOFTMAX(256, 4);
    else if (a.nk <= 4096)
        VSCAN_SOFTMAX(1024, 4);
    else if (a.nk <= 16384)
        VSCAN_SOFTMAX(1024, 16);
    else
        hipLaunchKernelGGL(fused_softmax_long_kernel, grid, dim3(1024), 0, s, a.c_l, a.ks_l,
                           ks_stride, a.nk, a.scale, a.Tq, a.causal, a.meta);
#undef VSCAN_SOFTMAX
    return hipGetLastError();
}

// 64 x 64 tiles of 16- or 32-bit elements through LDS (pitch 65: conflict-free both ways)
template <typename U>
__global__ __launch_bounds__(256) void transpose_kernel(const U *__restrict__ in, U *__restrict__ out,
                                                        int rows, int cols) {
    __shared__ U tile[64][65];
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
    for (int i = threadIdx.x; i < 64 * 64; i += 256) {
        const int r = i >> 6, c = i & 63;
        if (r0 + r < rows && c0 + c < cols) tile[r][c] = in[(int64_t)(r0 + r) * cols + c0 + c];
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 64 * 64; i += 256) {
        const int c = i >> 6, r = i & 63;
        if (r0 + r < rows && c0 + c < cols) out[(int64_t)(c0 + c) * rows + r0 + r] = tile[r][c];
    }
}

hipError_t launch_transpose(const void *in, void *out, int rows, int cols, int elem_bytes,
                            hipStream_t s) {
    const dim3 grid((cols + 63) / 64, (rows + 63) / 64);
    if (elem_bytes == 2)
        hipLaunchKernelGGL(transpose_kernel<uint16_t>, grid, dim3(256), 0, s, (const uint16_t *)in,
                           (uint16_t *)out, rows, cols);
    else
        hipLaunchKernelGGL(transpose_kernel<uint32_t>, grid, dim3(256), 0, s, (const uint32_t *)in,
                           (uint32_t *)out, rows, cols);
    return hipGetLastError();
}

template <typename T>
static hipError_t fused_project_t(const ProjectArgs &a, hipStream_t s) {
    ProbProject<T> pr;
    pr.d = dims(a.H * a.dh, a.BC * a.S, a.Dh, (int)sizeof(T), 1, nullptr);
    pr.hidden = reinterpret_cast<const char *>(a.hidden);
    pr.w = reinterpret_cast<const char *>(a.w);
    pr.S = a.S;
    pr.H = a.H;
    pr.dh = a.dh;
    pr.row_bytes = a.Dh * (int)sizeof(T);
    pr.out = a.out;
    return launch_gemm(pr, 1, s);
}
hipError_t launch_fused_project(const ProjectArgs &a, hipStream_t s) {
    return a.is_bf16 ? fused_project_t<bf16_t>(a, s) : fused_project_t<float>(a, s);
}

hipError_t launch_fused_colsum(const FusedArgs &a, hipStream_t s) {
    hipLaunchKernelGGL(fused_colsum_kernel, dim3((a.nk + 63) / 64, a.B), dim3(256), 0, s, a.c_l,
                       a.Hq * a.Tq, a.nk, a.vis_start - a.k0, a.V, a.causal, a.meta, a.part);
    return hipGetLastError();
}

}  // namespace vscan
