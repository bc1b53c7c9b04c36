// bf16-only building blocks of the tuned kernels (gfx950): LDS transpose reads, packed
// conversions, register-staged tile prefetch.
#pragma once
#include "lss_common.h"

namespace lss {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// DS_READ_B64_TR_B16: within each group of 16 lanes, lane i receives element (i % 4) of the
// 8-byte rows addressed by lanes (i / 4) + 4 * t, t = 0..3.  With lane s of a group addressing
// row (s / 4), 4-element column chunk (s % 4) of a row-major tile, lane i ends up with column i
// of 4 consecutive rows: a 4 x 16 block read transposed.
//
// tr_lane_offset(): element offset (within a row-major tile of `pitch` elements per row) that
// this lane passes so that, over the two reads of load_frag_tr, it receives for tile column
// (lane % 32) the 8 rows  8*a + 4*(lane/32) + t  (a = 0, 1; t = 0..3) -- exactly the rows that
// slots 4*a + t of a C-tile half carry (see lss_common.h).
__device__ __forceinline__ int tr_lane_offset(int lane, int pitch)
{
    const int grp = lane >> 4, hh = grp >> 1, nh = grp & 1, s = lane & 15;
    return (4 * hh + (s >> 2)) * pitch + 16 * nh + 4 * (s & 3);
}

// A-operand fragment of the TRANSPOSE of a row-major LDS tile: rows [row0, row0+16) become the
// contraction slots, columns [col0, col0+32) the 32 rows of the operand.
__device__ __forceinline__ Frag<bf16_t> load_frag_tr(const bf16_t *tile, int pitch, int row0, int col0, int lane_off)
{
    const bf16_t *p = tile + row0 * pitch + col0 + lane_off;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + 8 * pitch));
    const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    Frag<bf16_t> f;
    f.v = __builtin_bit_cast(bf16x8, both);
    return f;
}

// Register-staged copy of a [ROWS][D] bf16 tile: issue the global loads early (fetch), store
// them to LDS later (commit).  256 threads; 16-byte chunks.  The loads are unconditional so that
// the compiler can count them (a load under a branch forces a full wait on every later use of
// any loaded register): rows >= rows_ok re-read row rows_ok - 1, and the kernels make sure such
// rows only ever meet weights that are exactly 0.  Needs rows_ok >= 1.
template <int D, int ROWS>
struct TileStage {
    static constexpr int CPR = D / 8;                 // 16-byte chunks per row
    static constexpr int N = ROWS * CPR / 256;        // chunks per thread
    static_assert(ROWS * CPR % 256 == 0, "tile must divide among 256 threads");
    f32x4 r[N];

    __device__ __forceinline__ void fetch(const bf16_t *__restrict__ g, int64_t row_stride, int rows_ok, int tid)
    {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int c = i * 256 + tid, row = min(c / CPR, rows_ok - 1), col = (c % CPR) * 8;
            r[i] = *reinterpret_cast<const f32x4 *>(g + row * row_stride + col);
        }
    }
    __device__ __forceinline__ void commit(bf16_t *lds, int pitch, int tid) const
    {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int c = i * 256 + tid, row = c / CPR, col = (c % CPR) * 8;
            *reinterpret_cast<f32x4 *>(lds + row * pitch + col) = r[i];
        }
    }
};

// Wait until every outstanding vector-memory load of this wave has returned.  Placed once before
// a main loop it also tells the compiler's wait-count insertion that nothing loaded earlier (Q
// fragments, K/V operands) is still pending, so that inside the loop it only ever waits for the
// loop's own prefetch loads, and only where they are consumed.
__device__ __forceinline__ void wait_vmem_all() { __builtin_amdgcn_s_waitcnt(0x0F70); }   // vmcnt(0), others untouched

// 4 floats -> 4 bf16 (round to nearest even), as one 8-byte value
__device__ __forceinline__ bf16x4 pack4(float a, float b, float c, float d)
{
    bf16x4 v;
    v[0] = (bf16_t)a; v[1] = (bf16_t)b; v[2] = (bf16_t)c; v[3] = (bf16_t)d;
    return v;
}

} // namespace lss
