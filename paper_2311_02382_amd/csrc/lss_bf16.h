// bf16-only building blocks of the tuned kernels (gfx950): direct global -> LDS tile loads into
// swizzled tiles, LDS transpose reads, packed conversions.
#pragma once
#include "lss_common.h"

namespace lss {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// Global -> LDS load without a register in between: lane i moves BYTES (4 or 16) bytes from
// g_uniform + voff to lds_uniform + i * BYTES.  Base pointers are wavefront-uniform, voff per lane.
// Completion is counted like any vector-memory load (wait_vmem_all(), then a barrier, before any
// wavefront reads the data).  Written as inline assembly on purpose: through the compiler builtin
// every later LDS read that the compiler cannot prove disjoint would wait for the load at once,
// which defeats loading a ring slot a whole loop iteration ahead.  M0 (the LDS address register of
// the instruction) is saved and restored.
template <int BYTES>
__device__ __forceinline__ void lds_dma(const void *g_uniform, uint32_t voff, const void *lds_uniform)
{
    static_assert(BYTES == 4 || BYTES == 16, "");
    const uint32_t lds_addr = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char *)lds_uniform;
    uint32_t saved;
    if (BYTES == 16)
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3\n\ts_mov_b32 m0, %0"
                     : "=&s"(saved) : "s"(lds_addr), "v"(voff), "s"(g_uniform) : "memory");
    else
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %2, %3\n\ts_mov_b32 m0, %0"
                     : "=&s"(saved) : "s"(lds_addr), "v"(voff), "s"(g_uniform) : "memory");
}

// Chunk permutation of a row-major LDS tile with D bf16 columns (D / 8 chunks of 16 bytes per row): chunk c
// of row r sits at chunk position c ^ tile_swizzle<D>(r).  The LDS has 64 banks of 4 bytes, i.e. 16
// chunk-wide bank groups.  D = 64 (rows of 128 bytes, two rows per pass over the banks): r & 7 -- the 16
// rows of one plain fragment read and the 8 rows x 4 chunks of one transposing read each spread evenly.
// D = 128 (a row covers all banks once): with r & 7 the 8 rows x 4 chunks of a transposing read fall on 4
// bank groups per half of the rows (4-way conflicts: 6.4 cycles per instruction measured against 3.2);
// ((r & 3) << 2) | ((r >> 2) & 3) is a bijection on 16 consecutive rows (plain reads) whose upper two
// bits take every value twice on 8 consecutive rows (transposing reads).
template <int D>
__device__ __forceinline__ int tile_swizzle(int r)
{
    static_assert(D == 64 || D == 128, "");
    return D == 64 ? (r & 7) : (((r & 3) << 2) | ((r >> 2) & 3));
}

// [ROWS][D] bf16 tile loaded global -> LDS directly (no registers in between), by WAVES wavefronts.
// One such load instruction moves 16 bytes per lane and writes the wavefront's 64 chunks back to
// back (1 KB), so rows cannot be padded; instead the 16-byte chunk c of row r sits at chunk
// position c ^ tile_swizzle<D>(r) of its row, which spreads a column of chunks over the LDS banks as
// padding would.  The permutation is applied on the global side: the lane that fills position p of
// row r fetches chunk p ^ tile_swizzle<D>(r).
template <int D, int ROWS, int WAVES = 4>
struct DirectTile {
    static constexpr int CPR = D / 8;                 // 16-byte chunks per row
    static constexpr int RPI = 64 / CPR;              // rows per load instruction of one wavefront
    static constexpr int NI = ROWS / RPI / WAVES;     // load instructions per wavefront
    static constexpr int BYTES = ROWS * D * 2;
    static_assert(ROWS % (RPI * WAVES) == 0, "tile must divide among the wavefronts");

    // global byte offsets (from the tile's first row) of this lane's chunks; rows >= rows_ok
    // re-read row rows_ok - 1 and chunks >= chunks_ok re-read chunk chunks_ok - 1 (the kernels mask
    // or discard what such rows and columns produce).  Load instruction i of wavefront `wave` fills
    // the 1 KB at byte (i * WAVES + wave) * 1024 of the tile.  Needs ROWS * row_stride * 2 < 2^32.
    static __device__ __forceinline__ void offsets(uint32_t (&off)[NI], int64_t row_stride, int rows_ok, int wave, int lane,
                                                   int chunks_ok = CPR)
    {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int row = (i * WAVES + wave) * RPI + lane / CPR, pos = lane % CPR;
            const int chunk = min(pos ^ tile_swizzle<D>(row), chunks_ok - 1);
            off[i] = ((uint32_t)min(row, rows_ok - 1) * (uint32_t)row_stride + (uint32_t)chunk * 8u) * 2u;
        }
    }
    // Issue the loads of two tensors' tiles with one set of offsets, the second tile following the
    // first in LDS (lds_tile + BYTES).  Base pointers, `lds_tile` and `wave` must be wavefront-uniform.
    // One assembly block (see lds_dma for why assembly), so that M0 is saved and restored once and
    // merely stepped by WAVES KB (one KB per wavefront) from load to load.
    static __device__ __forceinline__ void issue_pair(const bf16_t *g0_uniform, const bf16_t *g1_uniform,
                                                      const uint32_t (&off)[NI], char *lds_tile, int wave)
    {
        static_assert(NI == 2 || NI == 4, "");
        constexpr int STEP = WAVES * 1024;              // between two load instructions of one wavefront
        const uint32_t lds_addr = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char *)(lds_tile + wave * 1024);
        uint32_t saved;
        if constexpr (NI == 2) {
            asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\t"
                         "global_load_lds_dwordx4 %2, %4\n\ts_add_u32 m0, m0, %6\n\ts_nop 0\n\t"
                         "global_load_lds_dwordx4 %3, %4\n\ts_add_u32 m0, m0, %6\n\ts_nop 0\n\t"
                         "global_load_lds_dwordx4 %2, %5\n\ts_add_u32 m0, m0, %6\n\ts_nop 0\n\t"
                         "global_load_lds_dwordx4 %3, %5\n\ts_mov_b32 m0, %0"
                         : "=&s"(saved)
                         : "s"(lds_addr), "v"(off[0]), "v"(off[1]), "s"(g0_uniform), "s"(g1_uniform), "i"(STEP)
                         : "memory", "scc");
        } else {
            asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\t"
                         "global_load_lds_dwordx4 %2, %6\n\ts_add_u32 m0, m0, %8\n\ts_nop 0\n\t"
                         "global_load_lds_dwordx4 %3, %6\n\ts_add_u32 m0, m0, %8\n\ts_nop 0\n\t"
                         "global_load_lds_dwordx4 %4, %6\n\ts_add_u32 m0, m0, %8\n\ts_nop 0\n\t"
                         "global_load_lds_dwordx4 %5, %6\n\ts_add_u32 m0, m0, %8\n\ts_nop 0\n\t"
                         "global_load_lds_dwordx4 %2, %7\n\ts_add_u32 m0, m0, %8\n\ts_nop 0\n\t"
                         "global_load_lds_dwordx4 %3, %7\n\ts_add_u32 m0, m0, %8\n\ts_nop 0\n\t"
                         "global_load_lds_dwordx4 %4, %7\n\ts_add_u32 m0, m0, %8\n\ts_nop 0\n\t"
                         "global_load_lds_dwordx4 %5, %7\n\ts_mov_b32 m0, %0"
                         : "=&s"(saved)
                         : "s"(lds_addr), "v"(off[0]), "v"(off[1]), "v"(off[2]), "v"(off[3]), "s"(g0_uniform), "s"(g1_uniform),
                           "i"(STEP)
                         : "memory", "scc");
        }
    }
    // byte offset inside the tile of the 16-byte chunk c of row r
    static __device__ __forceinline__ int chunk_offset(int r, int c) { return r * (D * 2) + ((c ^ tile_swizzle<D>(r)) * 16); }
};

// DS_READ_B64_TR_B16: within each group of 16 lanes, lane i receives element (i % 4) of the
// 8-byte rows addressed by lanes (i / 4) + 4 * t, t = 0..3.  With lane s of a group addressing
// row (s / 4), 4-element column chunk (s % 4) of a row-major tile, lane i ends up with column i
// of 4 consecutive rows: a 4 x 16 block read transposed.  (Lane mapping measured on the GPU.)
//
// A-operand fragment of the TRANSPOSE of a DirectTile: rows [row0, row0+16) become the contraction
// slots, the 32 columns of block `db` the 32 rows of the operand.  `lane_off` is this lane's byte
// offset for that column block (tr_lane_offset_sw), `row0` a multiple of 16.  Over the two reads
// the lane receives, for tile column (lane % 32), the 8 rows 8*a + 4*(lane/32) + t (a = 0, 1;
// t = 0..3) -- exactly the rows that slots 4*a + t of a C-tile half carry (see lss_common.h).
template <int D>
__device__ __forceinline__ Frag<bf16_t> load_frag_tr_sw(const char *tile, int row0, int lane_off)
{
    // the second read's rows lie 8 further down: the same permutation for D = 64, chunk position ^ 2 for D = 128
    const char *p = tile + row0 * (D * 2) + lane_off;
    const char *p8 = tile + row0 * (D * 2) + (D == 64 ? lane_off : (lane_off ^ 32)) + 8 * (D * 2);
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p8));
    const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    Frag<bf16_t> f;
    f.v = __builtin_bit_cast(bf16x8, both);
    return f;
}
// Byte offset for load_frag_tr_sw, columns [32 db, 32 db + 32): within its group of 16 lanes, lane
// s addresses row 4*hh + s/4 (+ row0, a multiple of 16, which does not change the permutation; + 8 for the
// second read, see load_frag_tr_sw) and the 8-byte piece (s % 4) of the 32-byte column group nh (hh,
// nh: bits 1 and 0 of the group index), at the position the chunk permutation of DirectTile gives it.
template <int D>
__device__ __forceinline__ int tr_lane_offset_sw(int lane, int db)
{
    const int grp = lane >> 4, hh = grp >> 1, nh = grp & 1, s = lane & 15;
    const int row = 4 * hh + (s >> 2), chunk = 4 * db + 2 * nh + ((s & 3) >> 1);
    return DirectTile<D, 64>::chunk_offset(row, chunk) + (s & 1) * 8;
}

// Workgroup order for grids of (batch*head, inner) work items.  Consecutive workgroup ids go to
// consecutive XCDs (8 of them, each with its own L2).  Item `id` is given batch*head
// bh = id % 8 + 8 * (id / 8 / n_inner) and inner index (id / 8) % n_inner: an XCD sees ONE head at
// a time (all inner items of head x, then of head x + 8, ...), so what the workgroups of a head
// share (K and V, or Q and dO) stays in that XCD's L2.  Grid size xcd_grid(bhs, n_inner); ids
// whose bh falls past bhs (bhs not a multiple of 8) have no work: xcd_item returns false.
constexpr int kXcds = 8;
inline int xcd_grid(int bhs, int n_inner) { return kXcds * ((bhs + kXcds - 1) / kXcds) * n_inner; }
__device__ __forceinline__ bool xcd_item(int id, int bhs, int n_inner, int &bh, int &inner)
{
    const int x = id % kXcds, rest = id / kXcds;
    inner = rest % n_inner;
    bh = x + kXcds * (rest / n_inner);
    return bh < bhs;
}

// Address of tile `tile` of a tensor whose tiles lie `tile_bytes` apart (below 2^32: 64 rows of at most 2^23
// elements): one 32 x 32 -> 64-bit scalar multiply and a 64-bit add, wavefront-uniform.
template <typename T>
__device__ __forceinline__ const T *tile_ptr(const T *base, int tile, uint32_t tile_bytes)
{
    return reinterpret_cast<const T *>(reinterpret_cast<const char *>(base) + (uint64_t)(uint32_t)tile * tile_bytes);
}

// Wait until every outstanding vector-memory load of this wave has returned, the direct
// global -> LDS ones included (their data is then in LDS; a barrier publishes it to the other
// wavefronts).
__device__ __forceinline__ void wait_vmem_all() { __builtin_amdgcn_s_waitcnt(0x0F70); }   // vmcnt(0), others untouched

// 4 floats -> 4 bf16 (round to nearest even), as one 8-byte value
__device__ __forceinline__ bf16x4 pack4(float a, float b, float c, float d)
{
    bf16x4 v;
    v[0] = (bf16_t)a; v[1] = (bf16_t)b; v[2] = (bf16_t)c; v[3] = (bf16_t)d;
    return v;
}

} // namespace lss
