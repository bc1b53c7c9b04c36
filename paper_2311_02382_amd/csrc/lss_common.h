// Device-side building blocks shared by the segment-attention kernels (gfx950).
//
// Matrix-core tile used throughout: V_MFMA_F32_32X32X16_BF16 (fp32 twin: eight
// V_MFMA_F32_32X32X2_F32).  One wavefront of 64 lanes computes a 32x32 fp32
// tile C += A(32x16) * B(16x32):
//   lane l holds, for A, row (l % 32), and for B, column (l % 32); both hold the 8
//   contraction slots of half (l / 32);
//   C is 16 floats per lane: element v is row 8*(v/4) + 4*(l/32) + (v%4), column l%32.
// A "fragment" below is one lane's 8 contraction slots.  Which contraction index a
// slot carries is free as long as A and B agree, which the kernels use to feed a C
// tile straight back in as a B operand: slots 8*s..8*s+7 of a C tile (s = 0, 1)
// carry rows 16*s + 8*(e/4) + 4*(l/32) + (e%4), e = 0..7.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lss {

typedef __bf16 bf16_t;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

template <typename T> struct Frag;
template <> struct Frag<bf16_t> { bf16x8 v; };
template <> struct Frag<float> { float v[8]; };

// C += A * B on the matrix cores, one 32x32x16 step.
__device__ __forceinline__ f32x16 mma(const Frag<bf16_t> &a, const Frag<bf16_t> &b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, b.v, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 mma(const Frag<float> &a, const Frag<float> &b, f32x16 c)
{
#pragma unroll
    for (int e = 0; e < 8; ++e) c = __builtin_amdgcn_mfma_f32_32x32x2f32(a.v[e], b.v[e], c, 0, 0, 0);
    return c;
}

// 8 consecutive elements (16-byte aligned for bf16, 32-byte span for float).
template <typename T> __device__ __forceinline__ Frag<T> load_frag(const T *p);
template <> __device__ __forceinline__ Frag<bf16_t> load_frag<bf16_t>(const bf16_t *p)
{
    Frag<bf16_t> f;
    f.v = *reinterpret_cast<const bf16x8 *>(p);
    return f;
}
template <> __device__ __forceinline__ Frag<float> load_frag<float>(const float *p)
{
    Frag<float> f;
    const f32x4 lo = *reinterpret_cast<const f32x4 *>(p);
    const f32x4 hi = *reinterpret_cast<const f32x4 *>(p + 4);
    f.v[0] = lo.x; f.v[1] = lo.y; f.v[2] = lo.z; f.v[3] = lo.w;
    f.v[4] = hi.x; f.v[5] = hi.y; f.v[6] = hi.z; f.v[7] = hi.w;
    return f;
}
template <typename T> __device__ __forceinline__ Frag<T> zero_frag();
template <> __device__ __forceinline__ Frag<bf16_t> zero_frag<bf16_t>()
{
    Frag<bf16_t> f;
#pragma unroll
    for (int e = 0; e < 8; ++e) f.v[e] = (bf16_t)0.0f;
    return f;
}
template <> __device__ __forceinline__ Frag<float> zero_frag<float>()
{
    Frag<float> f;
#pragma unroll
    for (int e = 0; e < 8; ++e) f.v[e] = 0.0f;
    return f;
}

// Slots 8*s..8*s+7 of a C tile as an operand fragment (rounded to nearest even for bf16).
template <typename T> __device__ __forceinline__ Frag<T> acc_to_frag(const f32x16 &c, int s);
template <> __device__ __forceinline__ Frag<bf16_t> acc_to_frag<bf16_t>(const f32x16 &c, int s)
{
    Frag<bf16_t> f;
#pragma unroll
    for (int e = 0; e < 8; ++e) f.v[e] = (bf16_t)c[8 * s + e];
    return f;
}
template <> __device__ __forceinline__ Frag<float> acc_to_frag<float>(const f32x16 &c, int s)
{
    Frag<float> f;
#pragma unroll
    for (int e = 0; e < 8; ++e) f.v[e] = c[8 * s + e];
    return f;
}

// Position of row x inside a transposed LDS tile: within each group of 16 rows the
// bits of weight 8 and 4 are swapped, so that the 8 rows one lane needs for a
// fragment built from a C tile (see the top of this file) are 8 consecutive elements.
__device__ __forceinline__ int tr_pos(int x)
{
    return (x & ~12) | ((x & 8) >> 1) | ((x & 4) << 1);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Dropout on the attention weights (Section 2.2), decided per weight from its position in the whole
// sequence, so that a segment drops what the sequential computation would drop there (Section 3,
// Principle 3): the weight of (batch*head bh, global query row, key col) is kept when
//     mix32(row key + column key) >= round(p * 2^32),
// where the row key mixes (low half of the seed, bh, row) and the column key (high half of the seed,
// col); mix32 is a published 32-bit mixing function (xorshift-multiply, two rounds).  No state, no
// stream.  The split into a row and a column key is what a kernel needs: one whose lanes own query
// rows keeps a row key per lane, one whose lanes own keys a column key per lane, and the other key
// of a tile's 64 rows or columns is computed once per tile.
__device__ __forceinline__ uint32_t mix32(uint32_t x)
{
    x = (x ^ (x >> 16)) * 0x7feb352du;
    x = (x ^ (x >> 15)) * 0x846ca68bu;
    return x ^ (x >> 16);
}
__device__ __forceinline__ uint32_t drop_row_key(uint32_t seed_lo, uint32_t bh, uint32_t row)
{
    return mix32(mix32(seed_lo + 0x9e3779b9u * (bh + 1u)) ^ row);
}
// `cs` = drop_col_seed(seed_hi), the same for every column
__device__ __forceinline__ uint32_t drop_col_seed(uint32_t seed_hi) { return mix32(seed_hi + 0x85ebca6bu); }
__device__ __forceinline__ uint32_t drop_col_key(uint32_t cs, uint32_t col) { return mix32(cs ^ col); }
__device__ __forceinline__ bool drop_keep(uint32_t row_key, uint32_t col_key, uint32_t thr)
{
    return mix32(row_key + col_key) >= thr;
}

template <typename T> struct Elems16 { static constexpr int n = 16 / sizeof(T); };

// Cooperative copy of a [ROWS][D] tile of a [*, H, D]-strided tensor into LDS by the
// whole workgroup (NT threads): row-major into `rm` (pitch PR) and/or transposed
// into `tr` (element (row, c) at tr[c * PT + tr_pos(row)]).  Rows >= rows_ok read as 0.
template <typename T, int D, int ROWS, int NT, int PR, int PT, bool ROWMAJOR, bool TRANSPOSED>
__device__ __forceinline__ void load_tile(const T *__restrict__ g, int64_t row_stride, int rows_ok,
                                          T *rm, T *tr, int tid)
{
    constexpr int E = Elems16<T>::n;        // elements per 16-byte chunk
    constexpr int CPR = D / E;              // chunks per row
    constexpr int CHUNKS = ROWS * CPR;
    static_assert(CHUNKS % NT == 0, "tile must divide among the threads");
#pragma unroll
    for (int it = 0; it < CHUNKS / NT; ++it) {
        const int c = it * NT + tid;
        const int row = c / CPR, col = (c % CPR) * E;
        f32x4 raw = {0.f, 0.f, 0.f, 0.f};
        if (row < rows_ok) raw = *reinterpret_cast<const f32x4 *>(g + row * row_stride + col);
        if (ROWMAJOR) *reinterpret_cast<f32x4 *>(rm + row * PR + col) = raw;
        if (TRANSPOSED) {
            const T *e = reinterpret_cast<const T *>(&raw);
            const int pos = tr_pos(row);
#pragma unroll
            for (int i = 0; i < E; ++i) tr[(col + i) * PT + pos] = e[i];
        }
    }
}

// Exact GeLU, u Phi(u), and its derivative Phi(u) + u phi(u) (Phi, phi: the standard normal's
// distribution function and density).
__device__ __forceinline__ float gelu_value(float u) { return u * (0.5f * (1.0f + erff(u * 0.70710678118654752f))); }
__device__ __forceinline__ float gelu_slope(float u)
{
    return 0.5f * (1.0f + erff(u * 0.70710678118654752f)) + u * 0.3989422804014327f * __expf(-0.5f * u * u);
}

} // namespace lss
