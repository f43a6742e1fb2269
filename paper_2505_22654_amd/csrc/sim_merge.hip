// Similarity-based token merging (Sec. 4.1 "Token Merging", Eq. 4).
//
//   sim_argmax      for every dropped token u: argmax_s (x_s . x_u) / ||x_s|| over
//                   the image's kept tokens.  ||x_u|| is a positive per-token
//                   constant and cannot change the argmax, so it is never formed;
//                   ||x_s|| is accumulated from the very tiles the GEMM stages.
//                   A kept x dropped GEMM on the matrix cores; the epilogue folds
//                   each column into a packed (similarity key, ~slot) word and
//                   merges it with atomicMax, which is order-independent and puts
//                   ties on the lowest slot.
//   merge           Eq. 4: one wave per kept slot averages the slot's own token
//                   and its members in ascending token order (fixed order: no
//                   floating-point atomics, bit-reproducible).
#include <atomic>

#include "common.hpp"
#include "launch.hpp"

namespace vscan {

constexpr float kNormEps = 1e-12f;

// ---------------------------------------------------------------------------
// kept x dropped similarity with fused norm and argmax.
// Workgroup tile: (64*TM) kept slots x (64*TN) dropped tokens, multiplied by 4 waves as 2 x 2,
// each wave TM x TN blocks of 32 x 32.  The feature axis is streamed through LDS in stages of
// KC 32-byte chunks, rows gathered by index.  NSETS stages are kept in flight in registers on
// top of the one being multiplied.  The small problems are a handful of stages long and give
// a CU one workgroup at most, so their time is set by how many memory round-trips are
// serialised, not by bandwidth: they run with 8 waves (the upper four only fetch), which halves
// the registers a stage costs per thread and lets four stages fly.  Large problems use one
// register set, so that two workgroups fit a CU and hide each other.
// ---------------------------------------------------------------------------
template <typename T, int TM, int TN, int KC, int NSETS, int THREADS>
__global__ __launch_bounds__(THREADS) void sim_argmax_kernel(const T *__restrict__ x,
                                                             const int32_t *__restrict__ kept_idx,
                                                             const int32_t *__restrict__ drop_idx,
                                                             unsigned long long *__restrict__ best,
                                                             int T_img, int D, int K, int U, int B,
                                                             int affine) {
    constexpr int E = ElemTraits<T>::kPer16B;
    constexpr int BM = 64 * TM, BN = 64 * TN, ROWS = BM + BN;
    constexpr int PPR = KC * 2;                 // 16-byte pieces per row per stage
    constexpr int STRIDE = KC * 32 + 16;        // LDS row stride in bytes
    constexpr int PER_THREAD = ROWS * PPR / THREADS;
    constexpr int A_PIECES = BM * PPR / THREADS;  // the first A_PIECES pieces of a thread are kept rows
    static_assert(ROWS * PPR % THREADS == 0 && BM * PPR % THREADS == 0, "tile must split evenly");
    static_assert(NSETS == 1 || NSETS == 2 || NSETS == 4, "register sets");
    static_assert(PPR <= 64 && (PPR & (PPR - 1)) == 0, "a row's pieces must sit in one wave");
    __shared__ __align__(16) unsigned char lds[2][ROWS * STRIDE];
    __shared__ __align__(16) float inv_s[BM];

    const int tiles_n = (U + BN - 1) / BN, tiles_m = (K + BM - 1) / BM;
    int b, tile;
    if (!image_affine_decode(B, tiles_m * tiles_n, affine != 0, b, tile)) return;
    const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;
    const int tid = threadIdx.x, lane = lane_id(), g = lane >> 5;
    const bool computes = THREADS == 256 || wave_id() < 4;  // waves 4.. (if any) only fetch
    const int wm = (wave_id() & 3) >> 1, wn = wave_id() & 1;
    const int row_bytes = D * (int)sizeof(T);
    const unsigned char *xb =
        reinterpret_cast<const unsigned char *>(x) + (int64_t)b * T_img * row_bytes;

    // byte offset of the row behind each piece this thread stages; 32 bits are enough: the ABI
    // layer rejects images of 2 GiB or more.  Rows outside the problem (slots >= K, columns
    // >= U) stage some other row of the image: their results are masked in the epilogue, and
    // a real row keeps every load unconditional and inside the image.
    int src[PER_THREAD];
    {
        // token of every row this thread stages.  Positions are clamped, not predicated: the
        // index loads stay independent of each other and are all in flight together.  A thread's
        // first A_PIECES pieces belong to kept rows, the rest to dropped rows.
        int tok[PER_THREAD];
#pragma unroll
        for (int it = 0; it < PER_THREAD; ++it) {
            const int r = (tid + it * THREADS) / PPR;
            tok[it] = it < A_PIECES ? kept_idx[(int64_t)b * K + min(m0 + r, K - 1)]
                                    : drop_idx[(int64_t)b * U + min(n0 + r - BM, U - 1)];
        }
#pragma unroll
        for (int it = 0; it < PER_THREAD; ++it)  // indices come from device memory: stay inside
            src[it] = min(max(tok[it], 0), T_img - 1) * row_bytes;
    }
    // dropped token of each result column this lane reports in the epilogue (fetched here so
    // that the latency is long gone by then)
    int col_tok[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = n0 + (wn * TN + j) * 32 + (lane & 31);
        col_tok[j] = drop_idx[(int64_t)b * U + min(col, U - 1)];
    }
    float ss[A_PIECES];  // partial squared norms of the kept rows this thread stages
#pragma unroll
    for (int it = 0; it < A_PIECES; ++it) ss[it] = 0.f;

    // Loads carry no condition (a piece past the end of the row re-reads the row's last piece
    // and is cleared when it is written to LDS), so the compiler can leave the loads of later
    // stages in flight while it waits for the stage it needs.
    auto stage_load = [&](int stage, uint4(&regs)[PER_THREAD]) {
#pragma unroll
        for (int it = 0; it < PER_THREAD; ++it) {
            const int piece = (tid + it * THREADS) % PPR;
            const int col_byte = min(stage * KC * 32 + piece * 16, row_bytes - 16);
            regs[it] = load16(xb, (int64_t)src[it] + col_byte);
        }
    };
    auto stage_store = [&](unsigned char *dst, const uint4(&regs)[PER_THREAD], int stage) {
#pragma unroll
        for (int it = 0; it < PER_THREAD; ++it) {
            const int p = tid + it * THREADS;
            const int r = p / PPR, piece = p - r * PPR;
            const uint4 val = stage * KC * 32 + piece * 16 < row_bytes ? regs[it] : zero16();
            *reinterpret_cast<uint4 *>(dst + r * STRIDE + piece * 16) = val;
            if (it < A_PIECES) {
                float v[E];
                unpack16<T>(val, v);
#pragma unroll
                for (int e = 0; e < E; ++e) ss[it] = fmaf(v[e], v[e], ss[it]);
            }
        }
    };

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    auto compute = [&](const unsigned char *cur) {
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
    };

    // Stage s sits in register set s % NSETS until it is written to LDS buffer s % 2, one
    // iteration before it is multiplied; the set is then refilled with stage s + NSETS.  (The
    // loop is unrolled by NSETS so that the sets are addressed statically.)
    const int nstages = (row_bytes + KC * 32 - 1) / (KC * 32);
    if constexpr (NSETS == 1) {
        uint4 ra[PER_THREAD];
        stage_load(0, ra);
        stage_store(lds[0], ra, 0);
        __syncthreads();
        for (int st = 0; st < nstages; ++st) {
            if (st + 1 < nstages) stage_load(st + 1, ra);
            if (computes) compute(lds[st & 1]);
            if (st + 1 < nstages) {
                stage_store(lds[(st + 1) & 1], ra, st + 1);
                __syncthreads();
            }
        }
    } else {
        uint4 regs[NSETS][PER_THREAD];
#pragma unroll
        for (int j = 0; j < NSETS; ++j)
            if (j < nstages) stage_load(j, regs[j]);
        stage_store(lds[0], regs[0], 0);
        __syncthreads();
        int st = 0;
        // groups in which every stage refills its register set: no condition around the loads,
        // so the wait before a stage is written to LDS leaves the later stages in flight
        for (; st + 2 * NSETS <= nstages; st += NSETS) {
#pragma unroll
            for (int j = 0; j < NSETS; ++j) {
                const int cur = st + j;
                stage_load(cur + NSETS, regs[j]);
                if (computes) compute(lds[cur & 1]);
                stage_store(lds[(cur + 1) & 1], regs[(j + 1) % NSETS], cur + 1);
                __syncthreads();
            }
        }
        for (; st < nstages; st += NSETS) {  // the last groups
#pragma unroll
            for (int j = 0; j < NSETS; ++j) {
                const int cur = st + j;
                if (cur < nstages) {
                    if (cur + NSETS < nstages) stage_load(cur + NSETS, regs[j]);
                    if (computes) compute(lds[cur & 1]);
                    if (cur + 1 < nstages) {
                        stage_store(lds[(cur + 1) & 1], regs[(j + 1) % NSETS], cur + 1);
                        __syncthreads();
                    }
                }
            }
        }
    }

    // 1 / max(||x_s||, eps): add the PPR partial sums of each kept row (adjacent lanes)
#pragma unroll
    for (int it = 0; it < A_PIECES; ++it) {
        const float v = group_sum<PPR>(ss[it]);
        const int p = tid + it * THREADS;
        if (p % PPR == 0) inv_s[p / PPR] = 1.0f / fmaxf(sqrtf(v), kNormEps);
    }
    __syncthreads();

    if (!computes) return;  // no barrier below
    // epilogue: acc[i][j][r] = x_slot . x_token with
    //   slot  = m0 + (wm*TM + i)*32 + acc_row(r),  token column = n0 + (wn*TN + j)*32 + lane%32
    // (inverse norms 16 bytes at a time and no bound check inside a full tile, as in the large
    // form below)
    const bool full = m0 + BM <= K;  // uniform over the workgroup
    float best_v[TN];
    int best_s[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        best_v[j] = -INFINITY;
        best_s[j] = -1;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        float inv[16];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 t =
                *reinterpret_cast<const float4 *>(inv_s + (wm * TM + i) * 32 + 8 * q + 4 * g);
            inv[4 * q] = t.x;
            inv[4 * q + 1] = t.y;
            inv[4 * q + 2] = t.z;
            inv[4 * q + 3] = t.w;
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int rl = (wm * TM + i) * 32 + acc_row(r);
            const bool valid = full || m0 + rl < K;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const float v = acc[i][j][r] * inv[r];
                // slots are visited in ascending order: strict > keeps the lowest on ties
                if (valid && v > best_v[j]) {  // (a finite v beats the initial -inf)
                    best_v[j] = v;
                    best_s[j] = m0 + rl;
                }
            }
        }
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        unsigned long long packed =
            best_s[j] < 0 ? 0ull
                          : (((unsigned long long)float_to_key(best_v[j])) << 32) |
                                (unsigned long long)(uint32_t)~(uint32_t)best_s[j];
        const unsigned long long other = __shfl_xor(packed, 32, kWave);
        if (other > packed) packed = other;
        const int col = n0 + (wn * TN + j) * 32 + (lane & 31);
        if (g == 0 && col < U && packed != 0ull) {
            const int tok = min(max(col_tok[j], 0), T_img - 1);
            atomicMax(best + (int64_t)b * T_img + tok, packed);
        }
    }
}

// ---------------------------------------------------------------------------
// 1 / max(||x_s||, eps) of every kept row, for the large form of the similarity kernel below:
// one wave per kept row.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void kept_inv_norm_kernel(const T *__restrict__ x,
                                                            const int32_t *__restrict__ kept_idx,
                                                            float *__restrict__ inv_norm, int T_img,
                                                            int D, int K, int B) {
    constexpr int E = ElemTraits<T>::kPer16B;
    const int row = blockIdx.x * 4 + wave_id();  // b * K + slot
    if (row >= B * K) return;
    const int b = row / K;
    const int tok = min(max(kept_idx[row], 0), T_img - 1);
    const unsigned char *xr =
        reinterpret_cast<const unsigned char *>(x) + ((int64_t)b * T_img + tok) * D * (int64_t)sizeof(T);
    const int npieces = D / E;
    float ss = 0.f;
    for (int p0 = 0; p0 < npieces; p0 += 4 * kWave) {
        uint4 raw[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)  // clamped, not predicated: four independent loads in flight
            raw[u] = load16(xr, (int64_t)min(p0 + u * kWave + lane_id(), npieces - 1) * 16);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float v[E];
            unpack16<T>(raw[u], v);
            float part = 0.f;
#pragma unroll
            for (int e = 0; e < E; ++e) part = fmaf(v[e], v[e], part);
            ss += p0 + u * kWave + lane_id() < npieces ? part : 0.f;
        }
    }
    ss = wave_sum(ss);
    if (lane_id() == 0) inv_norm[row] = 1.0f / fmaxf(sqrtf(ss), kNormEps);
}

// 16-byte loads from global memory straight into LDS: lane l's data lands 16*l bytes behind the
// wave-uniform LDS address held in M0; the source is a wave-uniform base plus a per-lane unsigned
// 32-bit byte offset.  Issued from inline assembly so that the compiler's wait-count bookkeeping
// does not see them (it would make every LDS read wait for them, whichever buffer they fill); the
// kernel waits for them itself before the barrier that publishes a stage.  (M0 is a reserved
// register that compiler-generated code loads right before each instruction that reads it and
// that these kernels use for nothing else.)
__device__ __forceinline__ unsigned lds_byte_address(const void *p) {
    return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}
__device__ __forceinline__ void direct_load16(const void *base, uint32_t byte_offset,
                                              unsigned lds_address) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_address), "v"(byte_offset), "s"(base)
                 : "memory");
}
// every outstanding vector-memory load of this wave has arrived (vmcnt 0, other counters left alone)
__device__ __forceinline__ void wait_direct_loads() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// ---------------------------------------------------------------------------
// The large form of the kept x dropped similarity: 128 x 128 workgroup tiles of 2 x 2 waves.
// Counters on the form above showed fifteen vector instructions per matrix instruction at this
// size (squared norms of the staged kept rows, 64-bit address arithmetic and clamps for every
// 16-byte piece and stage), which made the vector ALU, not the matrix cores, the busiest unit.
// Here the inverse norms come precomputed (kept_inv_norm_kernel) and a stage's loads use buffer
// addressing - the image in a resource descriptor, per-thread 32-bit offsets fixed for the
// whole kernel, the stage's column offset in a scalar register: no vector arithmetic per load.
// ---------------------------------------------------------------------------
// Workgroup tile (32 TM WM) kept slots x (32 TN WN) dropped tokens, WM x WN waves of TM x TN
// blocks.  Two shapes are used: 128 x 128 with four waves, two workgroups per CU (kept sets of
// a few hundred slots, where larger tiles would be mostly padding), and 256 x 256 with eight
// waves of 128 x 64 (one workgroup per CU), which halves the operand traffic from L2 into LDS
// per multiply-add and reads 0.75 operand fragments from LDS per matrix instruction instead of 1.
//
// Which tile a workgroup takes (`mode`): 0 = in launch order; 1 = images pinned to XCDs (eight
// or more images: image_affine_decode); 2 = one large image: workgroups are handed to the 8 XCDs
// round-robin by linear index and every XCD has its own L2, so XCD x works through a compact
// block of (tiles_m / 4) x (tiles_n / 2) tiles, kept tile fastest - its band of kept rows stays
// in its L2 and its band of dropped rows streams through once.
template <typename T, int TM, int TN, int WM, int WN, int KC, int NSETS, bool DIRECT>
__global__ __launch_bounds__(64 * WM * WN, (WM * WN <= 4 && TM * TN <= 4) ? 2 : 1) void sim_argmax_large_kernel(
    const T *__restrict__ x, const int32_t *__restrict__ kept_idx,
    const int32_t *__restrict__ drop_idx, const float *__restrict__ inv_norm,
    unsigned long long *__restrict__ best, int T_img, int D, int K, int U, int B, int mode) {
    constexpr int THREADS = 64 * WM * WN;
    constexpr int BM = 32 * TM * WM, BN = 32 * TN * WN, ROWS = BM + BN;
    constexpr int PPR = KC * 2;                 // 16-byte pieces per row per stage
    // LDS row stride in bytes.  Staged through registers: 16 bytes of padding per row make the
    // 16-byte operand reads conflict-free.  DIRECT (stages fetched straight into LDS, which
    // writes a wave's 64 pieces contiguously and so leaves no room for padding): 128-byte rows
    // whose 16-byte columns are XOR-ed with the row's low three bits instead (86 % of the LDS
    // read rate, measured).
    static_assert(!DIRECT || KC == 4, "the column swizzle is written for rows of eight pieces");
    constexpr int STRIDE = DIRECT ? KC * 32 : KC * 32 + 16;
    constexpr int PER_THREAD = ROWS * PPR / THREADS;
    constexpr int A_PIECES = BM * PPR / THREADS;
    static_assert(ROWS * PPR % THREADS == 0 && BM * PPR % THREADS == 0, "tile must split evenly");
    static_assert(THREADS % PPR == 0, "a thread keeps its piece column for all its rows");
    extern __shared__ __align__(16) unsigned char lds_raw[];  // two stages, then BM inverse norms
    unsigned char(*lds)[ROWS * STRIDE] = reinterpret_cast<unsigned char(*)[ROWS * STRIDE]>(lds_raw);
    float *inv_s = reinterpret_cast<float *>(lds_raw + 2 * ROWS * STRIDE);

    const int tiles_n = (U + BN - 1) / BN, tiles_m = (K + BM - 1) / BM;
    int b, tile_m, tile_n;
    if (mode == 2) {
        const int id = blockIdx.x % (tiles_m * tiles_n);
        b = blockIdx.x / (tiles_m * tiles_n);
        const int xcd = id % kXcds, j = id / kXcds;          // j-th tile of this XCD
        const int bm = tiles_m / 4, bn = tiles_n / 2;         // the XCD's block of tiles
        tile_m = (xcd % 4) * bm + j % bm;
        tile_n = (xcd / 4) * bn + j / bm;
    } else {
        int tile;
        if (!image_affine_decode(B, tiles_m * tiles_n, mode == 1, b, tile)) return;
        tile_m = tile / tiles_n;
        tile_n = tile - tile_m * tiles_n;
    }
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int tid = threadIdx.x, lane = lane_id(), g = lane >> 5;
    const int wm = wave_id() / WN, wn = wave_id() % WN;
    const int row_bytes = D * (int)sizeof(T);
    const unsigned char *xb =
        reinterpret_cast<const unsigned char *>(x) + (int64_t)b * T_img * row_bytes;

    // Byte offset, inside the image, of the piece column this thread carries in each of its
    // rows (32 bits: the ABI layer rejects images of 2 GiB or more).  Rows outside the problem
    // (slots >= K, columns >= U) stage some other row of the image: their results are masked
    // in the epilogue, and a real row keeps every load unconditional and inside the image.
    // this thread's place in its LDS rows is column tid % PPR; the piece of the row that belongs
    // there is that column, or with the swizzle that column XOR the row's low bits
    const int piece = DIRECT ? (tid % PPR) ^ ((tid / PPR) & 7) : tid % PPR;
    uint32_t src[PER_THREAD];
    {
        int tok[PER_THREAD];
#pragma unroll
        for (int it = 0; it < PER_THREAD; ++it) {  // clamped positions: all index loads in flight
            const int r = tid / PPR + it * (THREADS / PPR);
            tok[it] = it < A_PIECES ? kept_idx[(int64_t)b * K + min(m0 + r, K - 1)]
                                    : drop_idx[(int64_t)b * U + min(n0 + r - BM, U - 1)];
        }
#pragma unroll
        for (int it = 0; it < PER_THREAD; ++it)  // indices come from device memory: stay inside
            src[it] = (uint32_t)(min(max(tok[it], 0), T_img - 1) * row_bytes + piece * 16);
    }
    int col_tok[TN];  // dropped token of each result column this lane reports in the epilogue
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = n0 + (wn * TN + j) * 32 + (lane & 31);
        col_tok[j] = drop_idx[(int64_t)b * U + min(col, U - 1)];
    }
    for (int i = tid; i < BM; i += THREADS) inv_s[i] = inv_norm[(int64_t)b * K + min(m0 + i, K - 1)];

    const int nstages = (row_bytes + KC * 32 - 1) / (KC * 32);
    const int nfull = row_bytes / (KC * 32);  // stages that lie inside the row entirely
    // Buffer resource over this image (untyped 32-bit data format); every offset used with it
    // lies inside the image by construction, the hardware's range check is not relied upon.
    const __amdgpu_buffer_rsrc_t image = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<unsigned char *>(xb), 0, T_img * row_bytes, 0x00020000);
    auto stage_load = [&](int stage, uint4(&regs)[PER_THREAD]) {
        if (stage < nfull) {
            // buffer addressing: image base in the resource, the thread's fixed offset in a
            // vector register, the stage's column offset in a scalar register
            const int soff = stage * (KC * 32);
#pragma unroll
            for (int it = 0; it < PER_THREAD; ++it) {
                const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(image, (int)src[it], soff, 0);
                regs[it] = make_uint4(v.x, v.y, v.z, v.w);
            }
        } else {
            // the ragged last stage: a piece past the end of the row re-reads the row's last
            // piece and is cleared when it is written to LDS
#pragma unroll
            for (int it = 0; it < PER_THREAD; ++it) {
                const int col_byte = min(stage * KC * 32 + piece * 16, row_bytes - 16);
                regs[it] = load16(xb, (int64_t)(src[it] - piece * 16) + col_byte);
            }
        }
    };
    unsigned char *const my_lds = lds_raw + (tid / PPR) * STRIDE + (tid % PPR) * 16;
    auto stage_store = [&](int buf, const uint4(&regs)[PER_THREAD], int stage) {
        unsigned char *dst = my_lds + buf * (ROWS * STRIDE);
        if (stage < nfull) {  // uniform: the common case carries no per-piece selects
#pragma unroll
            for (int it = 0; it < PER_THREAD; ++it)
                *reinterpret_cast<uint4 *>(dst + it * (THREADS / PPR) * STRIDE) = regs[it];
        } else {
            const bool keep = stage * KC * 32 + piece * 16 < row_bytes;
#pragma unroll
            for (int it = 0; it < PER_THREAD; ++it)
                *reinterpret_cast<uint4 *>(dst + it * (THREADS / PPR) * STRIDE) =
                    keep ? regs[it] : zero16();
        }
    };

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // Operand fragments: two register sets, chunk c of a stage in set c & 1 (KC is even).  The
    // fragments of the next chunk are read from LDS before the matrix instructions of the
    // current one are issued - across the middle of a stage, and across the barrier at its end:
    // the first chunk of stage s + 1 is read right after the barrier and arrives under the
    // matrix instructions of stage s's last chunk.  No matrix instruction waits for LDS.
    static_assert(KC % 2 == 0, "chunk c lives in fragment set c & 1");
    const int a_off = (wm * 32 * TM + (lane & 31)) * STRIDE;
    const int b_off = (BM + wn * 32 * TN + (lane & 31)) * STRIDE;
    // byte offset of chunk c's 16 bytes inside a row (every row this lane reads has the same
    // low three bits as the lane: tiles and blocks start at multiples of 32)
    auto col_off = [&](int c) { return DIRECT ? 16 * ((g + 2 * c) ^ (lane & 7)) : 16 * g + 32 * c; };
    uint4 af[2][TM], bf[2][TN];
    auto read = [&](const unsigned char *cur, int c, int set) {
        const int co = col_off(c);
#pragma unroll
        for (int i = 0; i < TM; ++i)
            af[set][i] = *reinterpret_cast<const uint4 *>(cur + a_off + i * 32 * STRIDE + co);
#pragma unroll
        for (int j = 0; j < TN; ++j)
            bf[set][j] = *reinterpret_cast<const uint4 *>(cur + b_off + j * 32 * STRIDE + co);
    };
    auto mma = [&](int set) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) mma32_chunk<T>(acc[i][j], af[set][i], bf[set][j]);
    };

    // Stage s + 1 is written to the other LDS buffer in the middle of stage s (the LDS writes
    // complete under the second half of its matrix instructions), and the registers it came
    // from are refilled at once with the loads of stage s + 1 + NSETS: a load has NSETS whole
    // stages to arrive.  With one register set (the eight-wave form has no registers to spare)
    // that is one stage, about what a fetch from L2 takes while the chip is busy; the four-wave
    // form keeps three sets in flight.  Stage i always lives in set i % NSETS, so the loop is
    // unrolled NSETS times.
    if constexpr (DIRECT) {
        // Two LDS buffers, no staging registers: the loads of stage s + 1 are issued as soon as
        // the barrier at the end of stage s - 1 has freed its buffer, and have all of stage s
        // to arrive.  Rows that end inside a stage (the ragged last one) still pass through
        // registers, which clears what lies past their end; that one stage is fetched where it
        // is published, so its registers are not live across the matrix instructions.
        const unsigned lds0 = lds_byte_address(lds_raw);
        auto fetch = [&](int stage) {
            if (stage < nfull) {
                const unsigned char *sbase = xb + (int64_t)stage * (KC * 32);
#pragma unroll
                for (int it = 0; it < PER_THREAD; ++it)
                    direct_load16(sbase, src[it],
                                  __builtin_amdgcn_readfirstlane(
                                      lds0 + (unsigned)((stage & 1) * (ROWS * STRIDE) +
                                                        (it * (THREADS / PPR) + wave_id() * 8) * STRIDE)));
            }
        };
        auto publish = [&](int stage) {  // this wave's share of the stage is in LDS
            if (stage < nfull) {
                wait_direct_loads();
            } else {
                uint4 ra[PER_THREAD];
                stage_load(stage, ra);
                stage_store(stage & 1, ra, stage);
            }
        };
        fetch(0);
        publish(0);
        __syncthreads();
        read(lds[0], 0, 0);
        for (int st = 0; st < nstages; ++st) {
            const bool more = st + 1 < nstages;
            const unsigned char *cur = lds[st & 1];
            if (more) fetch(st + 1);
#pragma unroll
            for (int c = 0; c + 1 < KC; ++c) {
                read(cur, c + 1, (c + 1) & 1);
                mma(c & 1);
            }
            if (more) {
                publish(st + 1);
                __syncthreads();
                read(lds[(st + 1) & 1], 0, 0);
            }
            mma((KC - 1) & 1);
        }
    } else {
    uint4 ra[NSETS][PER_THREAD];
        stage_load(0, ra[0]);
        stage_store(0, ra[0], 0);
#pragma unroll
        for (int i = 1; i <= NSETS; ++i)
            if (i < nstages) stage_load(i, ra[i % NSETS]);
        __syncthreads();
        read(lds[0], 0, 0);
        for (int st0 = 0; st0 < nstages; st0 += NSETS) {
#pragma unroll
            for (int j = 0; j < NSETS; ++j) {
                const int st = st0 + j;
                if (st < nstages) {  // uniform
                    const bool more = st + 1 < nstages;
                    const int next_set = (j + 1) % NSETS;  // a constant once unrolled: st0 is a multiple of NSETS
                    const unsigned char *cur = lds[st & 1];
#pragma unroll
                    for (int c = 0; c + 1 < KC; ++c) {
                        read(cur, c + 1, (c + 1) & 1);
                        mma(c & 1);
                        if (c == KC / 2 - 1) {
                            if (more) stage_store((st + 1) & 1, ra[next_set], st + 1);
                            if (st + 1 + NSETS < nstages) stage_load(st + 1 + NSETS, ra[next_set]);
                        }
                    }
                    if (more) {
                        // every wave has issued its last reads of this buffer and its writes of the
                        // other one; both are complete when the barrier is passed
                        __syncthreads();
                        read(lds[(st + 1) & 1], 0, 0);
                    }
                    mma((KC - 1) & 1);
                }
            }
        }
    }

    // epilogue: acc[i][j][r] = x_slot . x_token with
    //   slot  = m0 + (wm*TM + i)*32 + acc_row(r),  token column = n0 + (wn*TN + j)*32 + lane%32
    // Registers 4q .. 4q+3 of a block are four consecutive slots, so their inverse norms come
    // from LDS 16 bytes at a time, once for all TN columns of blocks; a tile that lies wholly
    // inside the kept rows (every tile but a ragged last one) skips the per-slot bound check.
    // (With a 4-byte LDS read and a bound check per candidate the epilogue took 10.7 us of a
    // 256 x 256 tile's 51 us.)
    const bool full = m0 + BM <= K;  // uniform over the workgroup
    float best_v[TN];
    int best_s[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        best_v[j] = -INFINITY;
        best_s[j] = -1;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        float inv[16];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 t =
                *reinterpret_cast<const float4 *>(inv_s + (wm * TM + i) * 32 + 8 * q + 4 * g);
            inv[4 * q] = t.x;
            inv[4 * q + 1] = t.y;
            inv[4 * q + 2] = t.z;
            inv[4 * q + 3] = t.w;
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int rl = (wm * TM + i) * 32 + acc_row(r);
            const bool valid = full || m0 + rl < K;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const float v = acc[i][j][r] * inv[r];
                // slots are visited in ascending order: strict > keeps the lowest on ties
                if (valid && v > best_v[j]) {  // (a finite v beats the initial -inf)
                    best_v[j] = v;
                    best_s[j] = m0 + rl;
                }
            }
        }
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        unsigned long long packed =
            best_s[j] < 0 ? 0ull
                          : (((unsigned long long)float_to_key(best_v[j])) << 32) |
                                (unsigned long long)(uint32_t)~(uint32_t)best_s[j];
        const unsigned long long other = __shfl_xor(packed, 32, kWave);
        if (other > packed) packed = other;
        const int col = n0 + (wn * TN + j) * 32 + (lane & 31);
        if (g == 0 && col < U && packed != 0ull) {
            const int tok = min(max(col_tok[j], 0), T_img - 1);
            atomicMax(best + (int64_t)b * T_img + tok, packed);
        }
    }
}

// ---------------------------------------------------------------------------
// Eq. 4.  A workgroup of NW waves (4, or 16 for long images) owns NW * spw consecutive kept
// slots of one image.
//
// Phase 1 (whole workgroup): one pass over the image's assignment words; a token whose slot
// belongs to the workgroup is appended to that slot's member list in LDS (position from an LDS
// counter, so the order inside a list is arbitrary at this point).
// Phase 2 (one wave per slot, spw slots one after the other): the list is sorted by token index
// (rank by counting); a group of up to kMergeAloneCap members is added up by that wave right
// away, several rows in flight at a time (a shared group costs the workgroup two barriers and a
// pass over the partial sums, which is why groups of a few dozen are still added alone).
// Phase 3 (whole workgroup, one larger group after the other): group sizes are heavy-tailed
// (many dropped tokens look like the same kept token), and one wave adding dozens or hundreds
// of rows would set the kernel's time.  All waves share such a group: each takes its share of
// the sorted list - or, when the group is longer than the list, gathers the members inside its
// share of the token range with an ordered ballot scan - and the partial sums, one row per wave
// in LDS, are added column by column in wave order.
// Every sum has a fixed order of additions, so results do not depend on scheduling.
// Lane l owns the 16-byte pieces l, l+64, ... of the feature row.
// ---------------------------------------------------------------------------
constexpr int kMergeListCap = 128;  // ints of LDS per list

constexpr int kMergeAloneCap = 32;  // longest group that one wave adds alone (a few batches of rows)
constexpr int kMergeMaxSpw = 4;     // slots a wave handles one after the other, at most

template <typename T, int PIECES, int NW>
__global__ __launch_bounds__(64 * NW) void merge_kernel(const T *__restrict__ x,
                                                    const unsigned long long *__restrict__ best,
                                                    T *__restrict__ merged,
                                                    int32_t *__restrict__ assign_out, int T_img,
                                                    int D, int K, int B, int affine, int spw,
                                                    int parts, int part_pieces) {
    constexpr int E = ElemTraits<T>::kPer16B;
    // rows fetched together: about 24 16-byte loads per lane in flight (96 registers), which is
    // what it takes for the few workgroups that own the large groups to pull rows at the rate
    // a compute unit can take them
    // (sixteen waves share 512 registers per SIMD four ways: 128 each, so fewer rows per wave)
    constexpr int BATCH = NW == 16 ? (PIECES <= 1 ? 8 : PIECES == 2 ? 6 : PIECES == 3 ? 3 : 2)
                                   : (PIECES <= 3 ? 8 : PIECES <= 6 ? 4 : PIECES <= 12 ? 2 : 1);
    constexpr int NT = 64 * NW;       // threads
    __shared__ int cnt[NW * kMergeMaxSpw];
    __shared__ int lists[NW * kMergeMaxSpw][kMergeListCap];
    __shared__ int scratch_lists[NW][kMergeListCap];  // per wave, for the scans of phase 3
    extern __shared__ __align__(16) float part[];  // NW rows of part_pieces * E floats: partial sums
    const int ns = NW * spw;  // slots of this workgroup
    // `parts` workgroups share a set of slots: each adds the same rows, but only its own
    // `part_pieces` 16-byte columns of them (the last part may have fewer).  A group's rows are
    // added by one workgroup, on one compute unit, and the few groups of several hundred members
    // decide the kernel's time (10-20 us each); cut by columns, such a group is spread over
    // `parts` compute units with nothing to combine afterwards and the order of additions
    // untouched.  The price is that every part repeats the scan of the assignment words.
    int b, item;
    if (!image_affine_decode(B, ((K + ns - 1) / ns) * parts, affine != 0, b, item)) return;
    const int group = item / parts, col_part = item - group * parts;
    const int slot0 = group * ns;
    const int tid = threadIdx.x, lane = lane_id(), wave = wave_id();
    // low halves of the assignment words: the complemented slot of every token
    const uint32_t *slot_word = reinterpret_cast<const uint32_t *>(best + (int64_t)b * T_img);
    const unsigned char *xb = reinterpret_cast<const unsigned char *>(x) +
                              (int64_t)b * T_img * D * (int64_t)sizeof(T);
    const int piece0 = col_part * part_pieces;                   // first 16-byte column of this part
    const int npieces = min(D / E - piece0, part_pieces);     // and how many it has (>= 1)
    const int64_t row_bytes = (int64_t)D * sizeof(T);
    const int64_t col_bytes = (int64_t)piece0 * 16;

    if (tid < NW * kMergeMaxSpw) cnt[tid] = 0;
    __syncthreads();

    constexpr int SCAN = 8;  // assignment words fetched ahead per thread
    for (int base = 0; base < T_img; base += SCAN * NT) {
        // The index is clamped, not predicated: the loads stay independent of each other and
        // in flight together.
        uint32_t w[SCAN];
#pragma unroll
        for (int u = 0; u < SCAN; ++u) w[u] = slot_word[2 * min(base + u * NT + tid, T_img - 1)];
#pragma unroll
        for (int u = 0; u < SCAN; ++u) {
            const int t = base + u * NT + tid;
            const int s = (int)(~w[u]);
            const unsigned rel = (unsigned)(s - slot0);
            if (t < T_img && rel < (unsigned)ns && s < K) {
                const int pos = atomicAdd(&cnt[rel], 1);
                if (pos < kMergeListCap) lists[rel][pos] = t;
                if (assign_out && col_part == 0) assign_out[(int64_t)b * T_img + t] = s;
            }
        }
    }
    __syncthreads();

    float acc[PIECES][E];
    auto clear = [&]() {
#pragma unroll
        for (int p = 0; p < PIECES; ++p)
#pragma unroll
            for (int e = 0; e < E; ++e) acc[p][e] = 0.f;
    };
    // adds rows list[0 .. n) to acc, in list order.  BATCH rows are in flight all the time: as
    // soon as a row has been added, the row BATCH places further down the list is requested into
    // the registers it leaves (a wave that asked for a whole batch, waited, added and only then
    // asked for the next one spent 2-3 us per batch, a memory round-trip plus the additions).
    // No load carries a condition (a row past the end of the list re-reads the last member, a
    // piece past the end of the row its last piece): a load inside a branch makes the compiler
    // wait for all outstanding loads where the branch joins.
    auto drain = [&](const int *list, int n) {
        if (n <= 0) return;
        uint4 raw[BATCH][PIECES];
        auto fetch = [&](int j, int tok) {
            const int64_t row = tok * row_bytes + col_bytes;
#pragma unroll
            for (int p = 0; p < PIECES; ++p)
                raw[j][p] = load16(xb, row + (int64_t)min(lane + p * kWave, npieces - 1) * 16);
        };
        auto add = [&](int j) {
#pragma unroll
            for (int p = 0; p < PIECES; ++p) {
                float v[E];
                unpack16<T>(raw[j][p], v);
#pragma unroll
                for (int e = 0; e < E; ++e) acc[p][e] += v[e];
            }
        };
#pragma unroll
        for (int j = 0; j < BATCH; ++j) fetch(j, list[min(j, n - 1)]);
        int m = 0;
        for (; m + BATCH < n; m += BATCH) {  // rows m .. m+BATCH-1 are all members
            int next[BATCH];  // the next batch's tokens, read from LDS ahead of the additions
#pragma unroll
            for (int j = 0; j < BATCH; ++j) next[j] = list[min(m + BATCH + j, n - 1)];
#pragma unroll
            for (int j = 0; j < BATCH; ++j) {
                add(j);
                // the request reuses the registers the addition has just freed: keep the
                // scheduler from moving it (or a later row's) up, which would need new ones
                __builtin_amdgcn_sched_barrier(0);
                fetch(j, next[j]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int j = 0; j < BATCH; ++j)
            if (m + j < n) add(j);  // uniform over the wave
    };
    auto write_row = [&](int slot, int count) {
        const float inv = 1.0f / (float)count;
        unsigned char *out = reinterpret_cast<unsigned char *>(merged) +
                             ((int64_t)b * K + slot) * row_bytes + col_bytes;
#pragma unroll
        for (int p = 0; p < PIECES; ++p) {
            const int piece = lane + p * kWave;
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
                *reinterpret_cast<uint4 *>(out + (int64_t)piece * 16) = o;
            }
        }
    };

    // sorts list[0 .. count) ascending, count <= kMergeListCap: rank by counting, up to two
    // members per lane.  Only the calling wave touches the list; LDS operations of one wave
    // complete in order, so the reads are done before the write-back.
    auto sort_list = [&](int *list, int count) {
        const int v0 = lane < count ? list[lane] : 0x7fffffff;
        const int v1 = kWave + lane < count ? list[kWave + lane] : 0x7fffffff;
        int r0 = 0, r1 = 0;
        const int n0 = min(count, kWave);
        for (int j = 0; j < n0; ++j) {
            const int o = __builtin_amdgcn_readlane(v0, j);
            r0 += o < v0 ? 1 : 0;
            r1 += o < v1 ? 1 : 0;
        }
        for (int j = kWave; j < count; ++j) {
            const int o = __builtin_amdgcn_readlane(v1, j - kWave);
            r0 += o < v0 ? 1 : 0;
            r1 += o < v1 ? 1 : 0;
        }
        if (lane < count) list[r0] = v0;
        if (kWave + lane < count) list[r1] = v1;
    };

    // ---- phase 2: every wave sorts the lists of its slots and finishes the small groups
    bool any_shared = false;
    for (int i = 0; i < spw; ++i) {
        const int rel = wave + NW * i;
        const int slot = slot0 + rel;
        if (slot >= K) break;
        const int count = __builtin_amdgcn_readfirstlane(cnt[rel]);
        if (count > kMergeListCap) continue;  // list incomplete: gathered by a scan in phase 3
        int *list = lists[rel];
        sort_list(list, count);
        if (count > kMergeAloneCap) continue;
        clear();
        drain(list, count);
        write_row(slot, count);
    }
    for (int rel = 0; rel < ns; ++rel) any_shared |= slot0 + rel < K && cnt[rel] > kMergeAloneCap;
    if (!any_shared) return;  // the same decision in every wave: cnt is final since the barrier
    __syncthreads();          // sorted lists visible to all waves

    // ---- phase 3: larger groups, all waves on one group at a time
    const int share = ((T_img + NW * kWave - 1) / (NW * kWave)) * kWave;
    const int t_begin = min(T_img, wave * share), t_end = min(T_img, t_begin + share);
    int *scan_list = scratch_lists[wave];
    for (int rel = 0; rel < ns; ++rel) {
        const int slot = slot0 + rel;
        const int count = cnt[rel];
        if (slot >= K || count <= kMergeAloneCap) continue;  // uniform over the workgroup
        clear();
        if (count <= kMergeListCap) {
            // the sorted list is complete: wave w takes its w-th share
            const int per = (count + NW - 1) / NW;
            const int lo = min(wave * per, count), hi = min(lo + per, count);
            drain(lists[rel] + lo, hi - lo);
        } else {
            // too long for the list: wave w gathers the members inside the w-th share of the
            // token range with an ordered ballot scan
            int nlist = 0;
            for (int base = t_begin; base < t_end; base += SCAN * kWave) {
                uint32_t w[SCAN];
#pragma unroll
                for (int u = 0; u < SCAN; ++u)
                    w[u] = slot_word[2 * min(base + u * kWave + lane, T_img - 1)];
#pragma unroll
                for (int u = 0; u < SCAN; ++u) {
                    const int t = base + u * kWave + lane;
                    const bool mine = t < t_end && (int)(~w[u]) == slot;
                    const uint64_t mask = __ballot(mine);
                    if (mine) scan_list[nlist + __popcll(mask & lanemask_lt())] = t;
                    nlist += __popcll(mask);
                    if (nlist > kMergeListCap - kWave) {
                        drain(scan_list, nlist);
                        nlist = 0;
                    }
                }
            }
            drain(scan_list, nlist);
        }
        // Partial sums: every wave leaves its own in LDS (16-byte accesses, a row of
        // part_pieces * E floats per wave), then the workgroup's threads take four columns each
        // and add the waves' values in wave order - the same order on every run - scale, convert
        // and write them out.
        constexpr int Q = E / 4;  // float4 per 16-byte piece of the input
        const int wave_stride = part_pieces * Q;
        float4 *part4 = reinterpret_cast<float4 *>(part);
#pragma unroll
        for (int p = 0; p < PIECES; ++p) {
            const int piece = lane + p * kWave;
            if (piece < npieces) {
#pragma unroll
                for (int q = 0; q < Q; ++q)
                    part4[(size_t)wave * wave_stride + piece * Q + q] =
                        make_float4(acc[p][4 * q], acc[p][4 * q + 1], acc[p][4 * q + 2],
                                    acc[p][4 * q + 3]);
            }
        }
        __syncthreads();
        const float inv = 1.0f / (float)count;
        unsigned char *out = reinterpret_cast<unsigned char *>(merged) +
                             ((int64_t)b * K + slot) * row_bytes + col_bytes;
        for (int c = tid; c < npieces * Q; c += NT) {
            float4 sum = part4[c];
            for (int w = 1; w < NW; ++w) {
                const float4 v = part4[(size_t)w * wave_stride + c];
                sum.x += v.x;
                sum.y += v.y;
                sum.z += v.z;
                sum.w += v.w;
            }
            if constexpr (sizeof(T) == 4) {
                *reinterpret_cast<float4 *>(out + (int64_t)c * 16) =
                    make_float4(sum.x * inv, sum.y * inv, sum.z * inv, sum.w * inv);
            } else {
                uint2 o;
                o.x = f32_to_bf16_rne(sum.x * inv) | (f32_to_bf16_rne(sum.y * inv) << 16);
                o.y = f32_to_bf16_rne(sum.z * inv) | (f32_to_bf16_rne(sum.w * inv) << 16);
                *reinterpret_cast<uint2 *>(out + (int64_t)c * 8) = o;
            }
        }
        __syncthreads();  // the buffers are reused by the next shared group
    }
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
// Images are pinned to XCDs when there are enough of them to keep all eight busy and one
// XCD's share of the feature matrix has a chance to stay in its 4 MiB L2.
static bool image_affinity(const MergeArgs &a) {
    const int64_t image_bytes = (int64_t)a.T * a.D * (a.is_bf16 ? 2 : 4);
    const int per_xcd = (a.B + kXcds - 1) / kXcds;
    return a.B >= kXcds && per_xcd * image_bytes <= (int64_t)8 << 20;
}

template <typename T, int TM, int TN, int KC, int NSETS, int THREADS>
static hipError_t sim_t(const MergeArgs &a, hipStream_t s) {
    const int U = a.T - a.K;
    if (U <= 0) return hipSuccess;  // nothing was dropped: every token keeps its own slot
    const int tiles = ((U + 64 * TN - 1) / (64 * TN)) * ((a.K + 64 * TM - 1) / (64 * TM));
    const bool affine = image_affinity(a);
    dim3 grid(image_affine_grid(a.B, tiles, affine));
    hipLaunchKernelGGL((sim_argmax_kernel<T, TM, TN, KC, NSETS, THREADS>), grid, dim3(THREADS), 0, s,
                       (const T *)a.x, a.kept_idx, a.drop_idx, (unsigned long long *)a.best, a.T,
                       a.D, a.K, U, a.B, (int)affine);
    return hipGetLastError();
}
template <typename T, int TM, int TN, int WM, int WN, int KC, int NSETS, bool DIRECT>
static hipError_t sim_large_launch(const MergeArgs &a, hipStream_t s) {
    constexpr int BM = 32 * TM * WM, BN = 32 * TN * WN;
    const int U = a.T - a.K;
    const int tiles_m = (a.K + BM - 1) / BM, tiles_n = (U + BN - 1) / BN;
    const bool affine = image_affinity(a);
    const int mode = affine ? 1 : (tiles_m % 4 == 0 && tiles_n % 2 == 0 ? 2 : 0);
    const size_t smem = (size_t)2 * (BM + BN) * (KC * 32 + (DIRECT ? 0 : 16)) + BM * sizeof(float);
    auto kernel = sim_argmax_large_kernel<T, TM, TN, WM, WN, KC, NSETS, DIRECT>;
    static std::atomic<uint64_t> lds_allowed{0};
    if (smem > 64 * 1024) {
        hipError_t e = allow_large_lds(kernel, lds_allowed);
        if (e != hipSuccess) return e;
    }
    dim3 grid(image_affine_grid(a.B, tiles_m * tiles_n, affine));
    hipLaunchKernelGGL(kernel, grid, dim3(64 * WM * WN), smem, s, (const T *)a.x, a.kept_idx,
                       a.drop_idx, (const float *)a.inv_norm, (unsigned long long *)a.best, a.T,
                       a.D, a.K, U, a.B, mode);
    return hipGetLastError();
}

template <typename T>
static hipError_t sim_large_t(const MergeArgs &a, hipStream_t s) {
    hipLaunchKernelGGL(kept_inv_norm_kernel<T>, dim3((a.B * a.K + 3) / 4), dim3(256), 0, s,
                       (const T *)a.x, a.kept_idx, a.inv_norm, a.T, a.D, a.K, a.B);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // 256 x 256 tiles once both sides fill them and there are enough of them for every CU
    const int U = a.T - a.K;
    const long tiles256 = (long)(U / 256) * (a.K / 256) * a.B;
    if (a.K >= 1024 && U >= 1024 && tiles256 >= 2 * 256)
        return sim_large_launch<T, 4, 2, 2, 4, 4, 1, true>(a, s);
    return sim_large_launch<T, 2, 2, 2, 2, 4, 3, true>(a, s);
}

bool sim_argmax_uses_large_form(int B, int T, int K) {
    const int U = T - K;
    return (long)((U + 127) / 128) * ((K + 127) / 128) * B >= 400;
}

hipError_t launch_sim_argmax(const MergeArgs &a, hipStream_t s) {
    // large problems amortise operand traffic with 128 x 128 tiles; small ones need
    // the workgroup count of 64 x 64 tiles and long stages (few memory round-trips)
    if (a.T - a.K <= 0) return hipSuccess;  // nothing was dropped: every token keeps its own slot
    if (sim_argmax_uses_large_form(a.B, a.T, a.K))
        return a.is_bf16 ? sim_large_t<bf16_t>(a, s) : sim_large_t<float>(a, s);
    if (a.is_bf16) return sim_t<bf16_t, 1, 1, 8, 2, 512>(a, s);
    return sim_t<float, 1, 1, 8, 2, 512>(a, s);
}

template <typename T>
static hipError_t merge_t(const MergeArgs &a, hipStream_t s) {
    constexpr int E = ElemTraits<T>::kPer16B;
    const int all_pieces = a.D / E;
    // Rows of 128 and more 16-byte pieces are cut into two column halves, each added by a
    // workgroup of its own (config 3: 24.4 -> 20.9 us; three and four parts measured slower:
    // every part repeats the scan of the assignment words).
    int parts = all_pieces >= 2 * kWave ? 2 : 1;
    const bool affine = image_affinity(a);
    // Sixteen waves per workgroup for long images (from 8192 tokens) when rows are short enough
    // for sixteen partial-sum rows in LDS and there are slots for at least half the CUs: every
    // workgroup scans all assignment words of its image, and the few very large groups of such
    // an image set the kernel's time; both are then spread over four times as many waves
    // (config 4: 52.6 -> 39.2 us).  Shorter images measured slower that way (config 3: 28 -> 40
    // us with sixteen waves, no gain with eight): fewer, larger workgroups.
    // Such a workgroup has a CU to itself, so column halves would make a second round of
    // workgroups once there are more than the chip has CUs.
    const bool wide = all_pieces <= 3 * kWave && a.T >= 8192 && (int64_t)a.B * a.K >= 16 * 128;
    const int nw = wide ? 16 : 4;
    if (wide && (int64_t)a.B * ((a.K + 15) / 16) * parts > kCus) parts = 1;
    const int part_pieces = (all_pieces + parts - 1) / parts;  // >= 64 when halved: no empty part
    const int per_lane = (part_pieces + kWave - 1) / kWave;
    // slots per wave: one while that still gives every CU two workgroups of four waves (one of
    // sixteen); more for very many slots, where the shared scan is what has to be amortised
    int spw = 1;
    while (spw < kMergeMaxSpw && (int64_t)a.B * a.K >= (int64_t)nw * (wide ? 256 : 1024) * 2 * spw) spw *= 2;
    const int ns = nw * spw;
    dim3 grid(image_affine_grid(a.B, ((a.K + ns - 1) / ns) * parts, affine));
    // one row of a part's floats per wave: at most 64 KiB (four waves, 512 pieces)
    const size_t part_bytes = (size_t)nw * part_pieces * E * sizeof(float);
#define VSCAN_MERGE(P, NW)                                                                      \
    do {                                                                                        \
        static std::atomic<uint64_t> lds_allowed{0};                                            \
        if (part_bytes > 32 * 1024) { /* with the lists: more than the default 64 KiB */        \
            hipError_t e = allow_large_lds(merge_kernel<T, P, NW>, lds_allowed,                 \
                                           kMaxDynamicLds - NW * 3072 /* its static LDS */);    \
            if (e != hipSuccess) return e;                                                      \
        }                                                                                       \
        hipLaunchKernelGGL((merge_kernel<T, P, NW>), grid, dim3(64 * NW), part_bytes, s,        \
                           (const T *)a.x, (const unsigned long long *)a.best, (T *)a.merged,   \
                           a.assign_out, a.T, a.D, a.K, a.B, (int)affine, spw, parts,           \
                           part_pieces);                                                        \
    } while (0)
    if (wide) {
        if (per_lane <= 1) VSCAN_MERGE(1, 16);
        else if (per_lane <= 2) VSCAN_MERGE(2, 16);
        else VSCAN_MERGE(3, 16);
    } else if (per_lane <= 1) VSCAN_MERGE(1, 4);
    else if (per_lane <= 2) VSCAN_MERGE(2, 4);
    else if (per_lane <= 3) VSCAN_MERGE(3, 4);
    else if (per_lane <= 4) VSCAN_MERGE(4, 4);
    else if (per_lane <= 8) VSCAN_MERGE(8, 4);
    else if (per_lane <= 16) VSCAN_MERGE(16, 4);
    else return hipErrorInvalidValue;  // wider rows are rejected by the ABI layer
#undef VSCAN_MERGE
    return hipGetLastError();
}
hipError_t launch_merge(const MergeArgs &a, hipStream_t s) {
    return a.is_bf16 ? merge_t<bf16_t>(a, s) : merge_t<float>(a, s);
}

}  // namespace vscan
