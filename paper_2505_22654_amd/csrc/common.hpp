// Device-side building blocks shared by the VScan kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vscan {

constexpr int kWave = 64;

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

struct bf16_t {
    uint16_t bits;
};

template <typename T>
struct ElemTraits;
template <>
struct ElemTraits<float> {
    static constexpr int kPer16B = 4;
};
template <>
struct ElemTraits<bf16_t> {
    static constexpr int kPer16B = 8;
};

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// round-to-nearest-even fp32 -> bf16 bits (finite inputs)
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// Unpack one 16-byte piece of a row into floats: 4 (fp32) or 8 (bf16) values.
template <typename T>
__device__ __forceinline__ void unpack16(const uint4 &raw, float *out);
template <>
__device__ __forceinline__ void unpack16<float>(const uint4 &raw, float *out) {
    out[0] = __uint_as_float(raw.x);
    out[1] = __uint_as_float(raw.y);
    out[2] = __uint_as_float(raw.z);
    out[3] = __uint_as_float(raw.w);
}
template <>
__device__ __forceinline__ void unpack16<bf16_t>(const uint4 &raw, float *out) {
    out[0] = bf16_lo(raw.x);
    out[1] = bf16_hi(raw.x);
    out[2] = bf16_lo(raw.y);
    out[3] = bf16_hi(raw.y);
    out[4] = bf16_lo(raw.z);
    out[5] = bf16_hi(raw.z);
    out[6] = bf16_lo(raw.w);
    out[7] = bf16_hi(raw.w);
}

template <typename T>
__device__ __forceinline__ float load_elem(const T *p);
template <>
__device__ __forceinline__ float load_elem<float>(const float *p) {
    return *p;
}
template <>
__device__ __forceinline__ float load_elem<bf16_t>(const bf16_t *p) {
    return __uint_as_float(((uint32_t)p->bits) << 16);
}

// Order-preserving map of a finite float onto uint32 (larger float -> larger key).
// Every real value maps to a key >= 1, so 0 can stand for "no candidate".
__device__ __forceinline__ uint32_t float_to_key(float f) {
    uint32_t u = (f == 0.f) ? 0u : __float_as_uint(f);  // -0 and +0 compare equal
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }

__device__ __forceinline__ uint64_t lanemask_lt() {
    return (1ull << lane_id()) - 1ull;
}


// Wave-wide integer sum through DPP row operations only (no LDS crossbar, no scalar
// round-trip per step); every lane gets the total.
__device__ __forceinline__ int wave_sum_dpp(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, true);   // quad_perm [1,0,3,2]
    v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, true);   // quad_perm [2,3,0,1]
    v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xf, 0xf, true);  // row_half_mirror
    v += __builtin_amdgcn_update_dpp(0, v, 0x140, 0xf, 0xf, true);  // row_mirror
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, true);  // row_bcast15 -> rows 1, 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, true);  // row_bcast31 -> rows 2, 3
    return __builtin_amdgcn_readlane(v, 63);
}

// Wave-wide unsigned maximum through DPP row operations; every lane gets the result.
__device__ __forceinline__ uint32_t wave_umax_dpp(uint32_t x) {
    int v = (int)x;
    auto mx = [](int a, int b) { return (int)max((uint32_t)a, (uint32_t)b); };
    v = mx(v, __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, true));   // quad_perm [1,0,3,2]
    v = mx(v, __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, true));   // quad_perm [2,3,0,1]
    v = mx(v, __builtin_amdgcn_update_dpp(0, v, 0x141, 0xf, 0xf, true));  // row_half_mirror
    v = mx(v, __builtin_amdgcn_update_dpp(0, v, 0x140, 0xf, 0xf, true));  // row_mirror
    v = mx(v, __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, true));  // row_bcast15 -> rows 1, 3
    v = mx(v, __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, true));  // row_bcast31 -> rows 2, 3
    return (uint32_t)__builtin_amdgcn_readlane(v, 63);
}

// Reduction over aligned groups of G adjacent lanes (G a power of two); every lane of a group
// gets the group's result.  Groups of up to 16 lanes use DPP row operations only (quad permutes,
// then the half-row and row mirrors: once the lanes of a quad, or of a half row, all hold the
// same partial result, the mirrored lane supplies the other half's); wider groups finish through
// the LDS crossbar.  The pairs combined at every step are those of an xor butterfly, so a sum is
// bit-identical to one.
template <int CTRL>
__device__ __forceinline__ float dpp_lane(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
template <int G, typename Op>
__device__ __forceinline__ float group_reduce(float v, Op op) {
    static_assert(G >= 1 && G <= 64 && (G & (G - 1)) == 0, "power of two up to the wave size");
    if constexpr (G >= 2) v = op(v, dpp_lane<0xB1>(v));    // quad_perm [1,0,3,2]
    if constexpr (G >= 4) v = op(v, dpp_lane<0x4E>(v));    // quad_perm [2,3,0,1]
    if constexpr (G >= 8) v = op(v, dpp_lane<0x141>(v));   // row_half_mirror
    if constexpr (G >= 16) v = op(v, dpp_lane<0x140>(v));  // row_mirror
    if constexpr (G >= 32) v = op(v, __shfl_xor(v, 16, kWave));
    if constexpr (G >= 64) v = op(v, __shfl_xor(v, 32, kWave));
    return v;
}
template <int G>
__device__ __forceinline__ float group_sum(float v) {
    return group_reduce<G>(v, [](float a, float b) { return a + b; });
}
__device__ __forceinline__ float wave_max(float v) {
    return group_reduce<kWave>(v, [](float a, float b) { return fmaxf(a, b); });
}
__device__ __forceinline__ float wave_sum(float v) { return group_sum<kWave>(v); }

// Block-wide reductions through a small LDS buffer (>= 16 floats); every thread
// gets the result.  Order of combination is fixed, so results are reproducible.
__device__ __forceinline__ float block_max(float v, float *red) {
    v = wave_max(v);
    __syncthreads();
    if (lane_id() == 0) red[wave_id()] = v;
    __syncthreads();
    const int nw = (blockDim.x + kWave - 1) / kWave;
    float r = red[0];
    for (int w = 1; w < nw; ++w) r = fmaxf(r, red[w]);
    return r;
}
__device__ __forceinline__ float block_sum(float v, float *red) {
    v = wave_sum(v);
    __syncthreads();
    if (lane_id() == 0) red[wave_id()] = v;
    __syncthreads();
    const int nw = (blockDim.x + kWave - 1) / kWave;
    float r = red[0];
    for (int w = 1; w < nw; ++w) r += red[w];
    return r;
}

// ---------------------------------------------------------------------------
// 32x32 matrix-core tile, fed 32 bytes of the contraction axis at a time.
//
// A "chunk" is 32 consecutive bytes of a row (16 bf16 or 8 fp32).  Lane l holds
// the 16 bytes [16*(l/32), 16*(l/32)+16) of the chunk for row (l % 32) of its
// operand; both operands use the same split, so the contraction order inside a
// chunk is irrelevant.  Accumulator layout (D = A * B^T over rows):
//   acc[r] = D[i][j],  i = 8*(r/4) + 4*(l/32) + (r%4)  (row of A),  j = l % 32
//   (row of B).
// ---------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void mma32_chunk(f32x16_t &acc, const uint4 &a, const uint4 &b);

template <>
__device__ __forceinline__ void mma32_chunk<bf16_t>(f32x16_t &acc, const uint4 &a,
                                                    const uint4 &b) {
    union {
        uint4 u;
        bf16x8_t v;
    } ua, ub;
    ua.u = a;
    ub.u = b;
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ua.v, ub.v, acc, 0, 0, 0);
}

template <>
__device__ __forceinline__ void mma32_chunk<float>(f32x16_t &acc, const uint4 &a,
                                                   const uint4 &b) {
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0,
                                               0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0,
                                               0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0,
                                               0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0,
                                               0, 0);
}

__device__ __forceinline__ int acc_row(int r) {
    return 8 * (r >> 2) + 4 * (lane_id() >> 5) + (r & 3);
}

// ---------------------------------------------------------------------------
// 16x16 matrix-core tile, fed 64 bytes of the contraction axis at a time.
// Lane l holds bytes [16*(l/16), 16*(l/16)+16) of the 64-byte chunk for row
// (l % 16) of its operand.  acc[r] = D[i][j], i = 4*(l/16) + r (row of A),
// j = l % 16 (row of B).
// ---------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void mma16_chunk(f32x4_t &acc, const uint4 &a, const uint4 &b);

template <>
__device__ __forceinline__ void mma16_chunk<bf16_t>(f32x4_t &acc, const uint4 &a,
                                                    const uint4 &b) {
    union {
        uint4 u;
        bf16x8_t v;
    } ua, ub;
    ua.u = a;
    ub.u = b;
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ua.v, ub.v, acc, 0, 0, 0);
}

template <>
__device__ __forceinline__ void mma16_chunk<float>(f32x4_t &acc, const uint4 &a, const uint4 &b) {
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0,
                                               0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0,
                                               0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0,
                                               0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0,
                                               0, 0);
}

// ---------------------------------------------------------------------------
// Workgroup -> (image, item) mapping that keeps every image on one XCD.
// Workgroups are handed to the 8 XCDs round-robin by linear index, and each XCD
// has its own L2.  With `affine` set, image b is served only by XCD (b mod 8), so
// rows of its feature matrix that one kernel pulled into that L2 are still there
// for the next workgroup - and for the next kernel that maps images the same way.
// Grid size: image_affine_grid().  Returns false for a padding workgroup.
// ---------------------------------------------------------------------------
constexpr int kXcds = 8;
constexpr int kCus = 256;  // compute units of the MI355X
__host__ __device__ inline int image_affine_grid(int images, int per_image, bool affine) {
    return affine ? kXcds * ((images + kXcds - 1) / kXcds) * per_image : images * per_image;
}
__device__ __forceinline__ bool image_affine_decode(int images, int per_image, bool affine,
                                                    int &image, int &item) {
    const int id = blockIdx.x;
    if (affine) {
        const int j = id / kXcds;
        image = (id % kXcds) + kXcds * (j / per_image);
        item = j % per_image;
        return image < images;
    }
    image = id / per_image;
    item = id % per_image;
    return true;
}

__device__ __forceinline__ uint4 zero16() { return make_uint4(0u, 0u, 0u, 0u); }

// 16-byte global load, unconditional: the caller guarantees the address is readable (typically
// by clamping an index).  Loads that are not wrapped in a branch stay independent of each other,
// so the compiler can keep several in flight and wait only for the one it needs.
__device__ __forceinline__ uint4 load16(const void *base, int64_t byte_off) {
    return *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(base) + byte_off);
}

// Streaming variants (non-temporal hint) for data that is read once.  Measured on this GPU, a
// cold one-pass read runs markedly faster when its loads carry the hint.  (The compaction
// kernels keep plain loads and stores: there the hint helped only when nothing of the source
// was cache-resident, and hinted stores were slower throughout.)
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load16_stream(const void *base, int64_t byte_off) {
    const u32x4_t t = __builtin_nontemporal_load(
        reinterpret_cast<const u32x4_t *>(reinterpret_cast<const char *>(base) + byte_off));
    return make_uint4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ uint4 load16_stream_guard(const void *base, int64_t byte_off, bool valid) {
    if (!valid) return zero16();
    return load16_stream(base, byte_off);
}

// 16-byte global load, zero when `valid` is false (never touches memory then).
__device__ __forceinline__ uint4 load16_guard(const void *base, int64_t byte_off, bool valid) {
    if (!valid) return zero16();
    return *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(base) + byte_off);
}

}  // namespace vscan
