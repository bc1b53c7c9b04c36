// The linear maps either side of the segment attention, in the fused-communication form of
// Section 3, Principle 3 (Fig. 2(ii), (iii), (v)), as bf16 matrix-core GEMMs for gfx950:
//     forward   Q_i = x_i W_q (the segment's own rows),  [K | V] = x [W_k | W_v] (gathered sequence)
//     backward  dx_q = dQ_i W_q^T,  dx_partial = dK_part W_k^T + dV_part W_v^T
// dx_partial is what the segment sum (the reduce-scatter's arithmetic) then adds over segments.
//
// One kernel template computes C[m, n] = sum_k A[m, k] W'[k, n] for a short list of jobs.  A
// workgroup of eight wavefronts owns a 256 (m) x 256 (n) tile of C, held transposed in the
// accumulators (lane = row m of A, as the attention kernels hold one query per lane):
// C^T += W'^T A^T, so the weights are the A operand of the matrix instruction and the activations
// its B operand.  Each wavefront owns 128 (m) x 64 (n): 4 x 2 accumulator tiles, 8 matrix
// instructions per 6 operand fragments; two wavefronts share a SIMD, so one's LDS reads and barrier
// waits hide behind the other's matrix instructions.  The contraction runs in tiles of 64 through
// two LDS slots (64 KB each), the next tile loaded global -> LDS directly while the current one is
// multiplied; one barrier per tile.  The finished tile goes through LDS once more so that it is
// written to memory as whole rows.
//   W_TR   weights stored [k][n] (forward: W as given).  Their fragments come from the LDS tile
//          by transposing reads; otherwise the weights are stored [n][k] (backward: W as given
//          IS W'^T) and are read plainly.
//   OUT_F32  C is written as float (the backward maps, whose results are summed over segments
//          afterwards), else rounded once to bf16.
//   A_ANY  a job's A may be float (the dK/dV partials; `a_f32` of the job): rounded to bf16 on the
//          way into LDS, through registers; the contraction index runs over dK's columns, then
//          dV's.  Jobs with bf16 A (dQ) share the launch.
#include "lss_bf16.h"
#include "lss_kernels.h"

#include <mutex>
#include <type_traits>
#include <vector>

namespace lss {

namespace {

constexpr int PM = 256, PN = 256, PK = 64;      // workgroup tile, contraction tile
constexpr int P_WAVES = 8, P_NT = 64 * P_WAVES;
constexpr int P_ABYTES = PM * PK * 2, P_WBYTES = PN * PK * 2, P_SLOT = P_ABYTES + P_WBYTES;
constexpr int P_LDS = 2 * P_SLOT;               // 128 KB: one workgroup per compute unit

struct ProjJob {
    const void *a0, *a1;        // A: [batches][rows][lda]; a1 serves contraction indices >= k_split (or is unused)
    const bf16_t *w;            // weights, row stride ldw
    void *c0, *c1;              // C: [batches][rows][ldc]; columns >= n_split go to c1 (column n - n_split)
    int64_t a_batch_stride, c_batch_stride;     // elements
    int rows, rows_ok;          // rows per batch; leading rows of A that hold data (the rest count as 0)
    int batches, N, K, k_split, n_split, ldw;
    int a_f32;                  // A is float (only in kernels compiled with A_ANY)
    int wg_begin, m_tiles, n_tiles;             // first workgroup id of the job, tiles per batch, column tiles
};
// What happens to a finished bf16 tile on its way to memory (the feed-forward unit, whose GeLU
// would otherwise be a pass over memory of its own):
//   EPI_GELU       C is written to c0 and GeLU(C), of the rounded C, to c1 (same layout)
//   EPI_GELU_BWD   C, rounded, is multiplied by GeLU'(U) before it is written; U = a1, laid out like C
enum { EPI_NONE = 0, EPI_GELU = 1, EPI_GELU_BWD = 2 };

struct ProjArgs {
    ProjJob job[2];
    int n_jobs, lda, ldc, skip_tail;
};

using ATile = DirectTile<PK, PM, P_WAVES>;      // activations [256 m][64 k]
using WTile = DirectTile<PK, PN, P_WAVES>;      // weights [256 n][64 k]

// Weights [64 k][256 n], read transposed.  Loaded directly like a DirectTile, but its 512-byte rows
// all start at the same LDS bank, so the 16-byte chunk c of row r sits at chunk position
// c ^ 4 (r % 4): the eight rows that one transposing read touches (64 bytes of each) then spread
// evenly over the banks.
struct WTileTr {
    static constexpr int NI = PK * (PN / 8) / 64 / P_WAVES;     // load instructions per wavefront (2 rows each)
    // chunks >= chunks_ok (columns past the matrix) re-read chunk chunks_ok - 1; chunks_ok is a multiple of 8;
    // rows >= rows_ok re-read row rows_ok - 1
    static __device__ __forceinline__ void offsets(uint32_t (&off)[NI], int ldw, int wave, int lane, int chunks_ok,
                                                   int rows_ok = PK)
    {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int row = (i * P_WAVES + wave) * 2 + lane / 32, pos = lane % 32;
            const int chunk = min(pos ^ (4 * (row & 3)), chunks_ok - 1);
            off[i] = ((uint32_t)min(row, rows_ok - 1) * (uint32_t)ldw + (uint32_t)chunk * 8u) * 2u;
        }
    }
    // Transposing reads (see load_frag_tr_sw for the instruction's lane mapping): within its group
    // of 16 lanes, lane s addresses row 8 hh + s / 4 and the 8-byte piece s % 4 of the 32-byte
    // column group nh of column block db (hh, nh: bits 1 and 0 of the group index).
    static __device__ __forceinline__ int lane_offset(int lane, int db)
    {
        const int grp = lane >> 4, hh = grp >> 1, nh = grp & 1, s = lane & 15;
        const int row = 8 * hh + (s >> 2), chunk = 4 * db + 2 * nh + ((s & 3) >> 1);
        return row * (PN * 2) + ((chunk ^ (4 * (row & 3))) * 16) + (s & 1) * 8;
    }
    // A-operand fragment of the transposed tile for contraction step ks: operand row = column
    // (lane % 32) of block db, slot e = contraction index 16 ks + 8 hh + e -- the order in which a
    // plain 16-byte read delivers the other operand.
    static __device__ __forceinline__ Frag<bf16_t> load_frag(const char *tile, int ks, int lane_off)
    {
        const char *p = tile + ks * 16 * (PN * 2) + lane_off;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + 4 * (PN * 2)));
        const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        Frag<bf16_t> f;
        f.v = __builtin_bit_cast(bf16x8, both);
        return f;
    }
};

template <bool A_ANY, bool W_TR, bool OUT_F32, int EPI>
__global__ __launch_bounds__(P_NT, 1) void proj_gemm_kernel(ProjArgs args)
{
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    using OutT = typename std::conditional<OUT_F32, float, bf16_t>::type;
    static_assert(EPI == EPI_NONE || !OUT_F32, "the GeLU epilogues work on bf16 results");

    const int tid = threadIdx.x, lane = tid & 63, lq = lane & 31, hh = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;

    // ---- which tile: jobs back to back; inside a job consecutive ids go to consecutive XCDs, and an
    // XCD walks the column tiles of one row tile before the next, so the A rows it streams from HBM
    // are re-read from its own L2
    int ji = 0;
    if (args.n_jobs > 1 && (int)blockIdx.x >= args.job[1].wg_begin) ji = 1;
    const ProjJob &J = args.job[ji];
    const int id = blockIdx.x - J.wg_begin;
    const int slot_id = id / kXcds;
    const int n_tile = slot_id % J.n_tiles;
    const int bm = id % kXcds + kXcds * (slot_id / J.n_tiles);
    if (bm >= J.batches * J.m_tiles) return;
    const int batch = bm / J.m_tiles, m0 = (bm % J.m_tiles) * PM, n0 = n_tile * PN;

    const int rows_here = min(J.rows - m0, PM);                     // rows of C this tile owns
    const int rows_data = min(min(J.rows, J.rows_ok) - m0, PM);     // of which this many have data in A
    const int cols_here = min(J.N - n0, PN);                        // a multiple of 64

    // ---- the finished tile -> memory, through LDS so that whole rows are written: a pass covers
    // 16-byte chunks [0, 32) of every row (bf16: all 256 columns, one pass; float: 128 columns, two
    // passes); chunk c of row m sits at chunk position c ^ (m % 32) of the row's 512 bytes.
    // Accumulator tile (mb, nb), element v of this lane: row m = 128 wm + 32 mb + lq, columns
    // n = 64 wn + 32 nb + 8 (v / 4) + 4 hh + (v % 4).
    constexpr int CW = OUT_F32 ? 4 : 8;         // columns per 16-byte chunk
    constexpr int PASSES = OUT_F32 ? 2 : 1;
    auto store_tiles = [&](const f32x16 (&acc)[4][2], bool from_acc) {
        OutT *c0 = static_cast<OutT *>(J.c0) + (int64_t)batch * J.c_batch_stride + (int64_t)m0 * args.ldc;
        OutT *c1 = static_cast<OutT *>(J.c1) + (int64_t)batch * J.c_batch_stride + (int64_t)m0 * args.ldc;
#pragma unroll
        for (int pass = 0; pass < PASSES; ++pass) {
            if (from_acc) {
                __syncthreads();        // every wavefront is done with what the LDS held
                if (!OUT_F32 || (wn >> 1) == pass) {
#pragma unroll
                    for (int mb = 0; mb < 4; ++mb) {
                        const int m = 128 * wm + 32 * mb + lq;
                        const bool data = m < rows_data;
                        char *row = smem + m * 512;
#pragma unroll
                        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                            for (int g = 0; g < 4; ++g) {
                                f32x4 val = {0.f, 0.f, 0.f, 0.f};
                                if (data) val = f32x4{acc[mb][nb][4 * g], acc[mb][nb][4 * g + 1], acc[mb][nb][4 * g + 2], acc[mb][nb][4 * g + 3]};
                                if constexpr (OUT_F32) {
                                    const int c = 16 * (wn & 1) + 8 * nb + 2 * g + hh;
                                    *reinterpret_cast<f32x4 *>(row + ((c ^ (m & 31)) * 16)) = val;
                                } else {
                                    const int c = 8 * wn + 4 * nb + g;
                                    *reinterpret_cast<bf16x4 *>(row + ((c ^ (m & 31)) * 16) + hh * 8) = pack4(val[0], val[1], val[2], val[3]);
                                }
                            }
                    }
                }
                __syncthreads();
            }
            // thread tid: chunk tid % 32 of rows tid / 32, + 16, ...
            const int c = tid & 31;
            const int n = n0 + pass * 128 + c * CW;         // column of C; a chunk never straddles n_split
            const bool col_ok = pass * 128 + c * CW < cols_here;
            OutT *dst = n < J.n_split ? c0 + n : c1 + (n - J.n_split);
#pragma unroll
            for (int i = 0; i < PM / 16; ++i) {
                const int m = i * 16 + (tid >> 5);
                f32x4 raw = {0.f, 0.f, 0.f, 0.f};
                if (from_acc) raw = *reinterpret_cast<const f32x4 *>(smem + m * 512 + ((c ^ (m & 31)) * 16));
                if (col_ok && m < rows_here) {
                    if constexpr (EPI == EPI_GELU_BWD) {
                        const bf16_t *u = static_cast<const bf16_t *>(J.a1) + (int64_t)batch * J.c_batch_stride + (int64_t)(m0 + m) * args.ldc + n;
                        const bf16x8 uu = *reinterpret_cast<const bf16x8 *>(u);
                        bf16x8 cv = __builtin_bit_cast(bf16x8, raw);
#pragma unroll
                        for (int e = 0; e < 8; ++e) cv[e] = (bf16_t)((float)cv[e] * gelu_slope((float)uu[e]));
                        raw = __builtin_bit_cast(f32x4, cv);
                    }
                    *reinterpret_cast<f32x4 *>(dst + (int64_t)m * args.ldc) = raw;
                    if constexpr (EPI == EPI_GELU) {
                        bf16x8 cv = __builtin_bit_cast(bf16x8, raw);
#pragma unroll
                        for (int e = 0; e < 8; ++e) cv[e] = (bf16_t)gelu_value((float)cv[e]);
                        *reinterpret_cast<bf16x8 *>(c1 + n + (int64_t)m * args.ldc) = cv;
                    }
                }
            }
        }
    };

    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16 acc[4][2];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) acc[mb][nb] = zero16;

    if (rows_data <= 0) {       // no row of this tile has data: its rows of C are zero
        if (!args.skip_tail) store_tiles(acc, false);
        return;
    }

    const int T = J.K / PK;
    const int t_split = J.k_split / PK;

    // ---- tile loads
    uint32_t offA[ATile::NI], offW[W_TR ? WTileTr::NI : WTile::NI];
    const bool a_f32 = A_ANY && J.a_f32 != 0;   // workgroup-uniform
    ATile::offsets(offA, args.lda, rows_data, wave, lane);
    if constexpr (W_TR) WTileTr::offsets(offW, J.ldw, wave, lane, cols_here / 8);
    else WTile::offsets(offW, J.ldw, cols_here, wave, lane);

    const char *a0 = static_cast<const char *>(J.a0), *a1 = static_cast<const char *>(J.a1);
    const int AE = a_f32 ? 4 : 2;               // bytes per element of A
    const int64_t a_tile0 = ((int64_t)batch * J.a_batch_stride + (int64_t)m0 * args.lda) * AE;
    auto a_src = [&](int t) -> const char * {   // first element of contraction tile t of this row tile
        return (t < t_split ? a0 + (int64_t)t * PK * AE : a1 + (int64_t)(t - t_split) * PK * AE) + a_tile0;
    };
    auto issue_w = [&](int t, int slot) {
        char *dst = smem + slot * P_SLOT + P_ABYTES;
        const bf16_t *src = W_TR ? J.w + (int64_t)t * PK * J.ldw + n0 : J.w + (int64_t)n0 * J.ldw + (int64_t)t * PK;
#pragma unroll
        for (int i = 0; i < (W_TR ? WTileTr::NI : WTile::NI); ++i) lds_dma<16>(src, offW[i], dst + (i * P_WAVES + wave) * 1024);
    };
    auto issue_a = [&](int t, int slot) {       // bf16 A: direct
        char *dst = smem + slot * P_SLOT;
        const char *src = a_src(t);
#pragma unroll
        for (int i = 0; i < ATile::NI; ++i) lds_dma<16>(src, offA[i], dst + (i * P_WAVES + wave) * 1024);
    };
    // float A: thread `tid` converts the 8-element chunks tid, tid + 512, ... of the tile
    // (chunk c is columns 8 (c % 8) .. + 7 of row c / 8) and writes them where the direct load would
    constexpr int FCH = PM * 8 / P_NT;          // chunks per thread
    f32x4 stage[A_ANY ? 2 * FCH : 1];
    auto fetch_a = [&](int t) {
        if constexpr (A_ANY) {
            const char *src = a_src(t);
#pragma unroll
            for (int i = 0; i < FCH; ++i) {
                const int c = i * P_NT + tid, row = min(c >> 3, rows_data - 1);
                const f32x4 *p = reinterpret_cast<const f32x4 *>(src + ((int64_t)row * args.lda + (c & 7) * 8) * 4);
                stage[2 * i] = p[0];       // (re-read from L2 by the workgroups of the other column tiles)
                stage[2 * i + 1] = p[1];
            }
        }
    };
    auto stash_a = [&](int slot) {
        if constexpr (A_ANY) {
            char *dst = smem + slot * P_SLOT;
#pragma unroll
            for (int i = 0; i < FCH; ++i) {
                const int c = i * P_NT + tid;
                bf16x8 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) { v[e] = (bf16_t)stage[2 * i][e]; v[4 + e] = (bf16_t)stage[2 * i + 1][e]; }
                *reinterpret_cast<bf16x8 *>(dst + ATile::chunk_offset(c >> 3, c & 7)) = v;
            }
        }
    };

    // ---- per-lane LDS offsets of the operand fragments of contraction step ks (16 indices): slot e
    // of a fragment carries index 16 ks + 8 hh + e
    int b_off[4][4];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int m = 128 * wm + 32 * mb + lq;
            b_off[mb][ks] = ATile::chunk_offset(m, 2 * ks + hh);
        }
    int w_off[2][4];            // plain weights: row n = 64 wn + 32 nb + lq, chunk 2 ks + hh
    int wt_off[2];              // transposed reads: column block 2 wn + nb
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        wt_off[nb] = WTileTr::lane_offset(lane, 2 * wn + nb);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) w_off[nb][ks] = WTile::chunk_offset(64 * wn + 32 * nb + lq, 2 * ks + hh);
    }
    // One contraction tile: four steps of 16 indices.  The six operand fragments of step ks + 1 are
    // requested from LDS before the eight matrix instructions of step ks are issued (two sets of
    // fragment registers), so a wavefront's matrix instructions wait for reads that are a whole step
    // old instead of for the ones just issued.
    struct Frags { Frag<bf16_t> fb[4], fw[2]; };
    auto load_frags = [&](const char *at, const char *wt, int ks, Frags &f) __attribute__((always_inline)) {
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
            if constexpr (W_TR) f.fw[nb] = WTileTr::load_frag(wt, ks, wt_off[nb]);
            else f.fw[nb] = load_frag<bf16_t>(reinterpret_cast<const bf16_t *>(wt + w_off[nb][ks]));
        }
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) f.fb[mb] = load_frag<bf16_t>(reinterpret_cast<const bf16_t *>(at + b_off[mb][ks]));
    };
    auto compute = [&](int slot) {
        const char *at = smem + slot * P_SLOT, *wt = at + P_ABYTES;
        Frags f[2];
        load_frags(at, wt, 0, f[0]);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if (ks + 1 < 4) load_frags(at, wt, ks + 1, f[(ks + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mb = 0; mb < 4; ++mb)
#pragma unroll
                for (int nb = 0; nb < 2; ++nb) acc[mb][nb] = mma(f[ks & 1].fw[nb], f[ks & 1].fb[mb], acc[mb][nb]);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- main loop: tile t is multiplied from slot t % 2 while tile t + 1 travels into the other slot
    // (last read during tile t - 1, which every wavefront left at the barrier)
    if (a_f32) {
        fetch_a(0);
        issue_w(0, 0);
        stash_a(0);
        if (T > 1) fetch_a(1);
        wait_vmem_all();
        __syncthreads();
        for (int t = 0; t < T; ++t) {
            const int slot = t & 1;
            if (t + 1 < T) issue_w(t + 1, slot ^ 1);
            compute(slot);
            if (t + 1 < T) stash_a(slot ^ 1);
            wait_vmem_all();
            if (t + 2 < T) fetch_a(t + 2);      // in flight across the barrier, stashed after tile t + 1
            __syncthreads();
        }
    } else {
        issue_a(0, 0); issue_w(0, 0);
        wait_vmem_all();
        __syncthreads();
        for (int t = 0; t < T; ++t) {
            const int slot = t & 1;
            if (t + 1 < T) { issue_a(t + 1, slot ^ 1); issue_w(t + 1, slot ^ 1); }
            compute(slot);
            wait_vmem_all();
            __syncthreads();
        }
    }
    store_tiles(acc, true);
}


// Weight gradient of a linear map: dW[k, n] = sum_r A[r, k] dC[r, n], the contraction running over
// the rows of both operands.  Both are therefore loaded as [64 rows][256 columns] tiles and read
// through transposing LDS reads (WTileTr); a workgroup owns a 256 (k) x 256 (n) tile of dW for one
// chunk of rows of one batch entry and writes it in fp32, to dW itself when there is a single chunk,
// else to that chunk's partial result, which a fixed-order sum adds up afterwards.  Same wavefront
// layout, two-slot ring and LDS-staged stores as proj_gemm_kernel.
//   DC_F32  dC is float and may come from two tensors side by side (the dK and dV partials): it is
//           rounded to bf16 on its way into LDS, through registers, as proj_gemm_kernel does for a
//           float A.
struct WgradArgs {
    const bf16_t *a;            // batch b, row r: a + b * a_batch_stride + r * lda  (K columns)
    const void *dc0, *dc1;      // dC: columns < n_split from dc0, the others from dc1 (column n - n_split); row stride ldc
    int64_t a_batch_stride, dc_batch_stride;    // elements
    float *out;                 // [splits][K][N]
    int rows;                   // rows of every batch entry
    int batches, K, N, n_split, lda, ldc;
    int chunk_rows;             // rows per split, a multiple of 64
    int splits_per_batch, m_tiles, n_tiles;
};

template <bool DC_F32>
__global__ __launch_bounds__(P_NT, 1) void wgrad_gemm_kernel(WgradArgs g)
{
    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const int tid = threadIdx.x, lane = tid & 63, lq = lane & 31, hh = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;

    // consecutive ids go to consecutive XCDs; an XCD walks the output tiles of one chunk of rows, so
    // that chunk's rows of A and dC are read from HBM once per XCD
    const int tiles = g.m_tiles * g.n_tiles, splits = g.batches * g.splits_per_batch;
    const int x = blockIdx.x % kXcds, rest = blockIdx.x / kXcds;
    const int tile = rest % tiles, split = x + kXcds * (rest / tiles);
    if (split >= splits) return;
    const int batch = split / g.splits_per_batch;
    const int m0 = (tile / g.n_tiles) * PM, n0 = (tile % g.n_tiles) * PN;
    const int r0 = (split % g.splits_per_batch) * g.chunk_rows, r1 = min(r0 + g.chunk_rows, g.rows);
    const int T = (r1 - r0 + PK - 1) / PK;          // >= 1: the host sizes the splits so
    const int tail = (r1 - r0) - (T - 1) * PK;      // rows of the last tile, 1 .. 64
    const int cols_m = min(g.K - m0, PM), cols_n = min(g.N - n0, PN);

    uint32_t offA[WTileTr::NI], offA_last[WTileTr::NI], offW[DC_F32 ? 1 : WTileTr::NI], offW_last[DC_F32 ? 1 : WTileTr::NI];
    WTileTr::offsets(offA, g.lda, wave, lane, cols_m / 8);
    WTileTr::offsets(offA_last, g.lda, wave, lane, cols_m / 8, tail);
    if constexpr (!DC_F32) {
        WTileTr::offsets(offW, g.ldc, wave, lane, cols_n / 8);
        WTileTr::offsets(offW_last, g.ldc, wave, lane, cols_n / 8, tail);
    }
    const bf16_t *a_base = g.a + (int64_t)batch * g.a_batch_stride + (int64_t)r0 * g.lda + m0;
    auto issue = [&](int t, int slot) {
        char *dst = smem + slot * P_SLOT;
        const bf16_t *pa = a_base + (int64_t)t * PK * g.lda;
        const bool last = t == T - 1;
#pragma unroll
        for (int i = 0; i < WTileTr::NI; ++i) lds_dma<16>(pa, last ? offA_last[i] : offA[i], dst + (i * P_WAVES + wave) * 1024);
        if constexpr (!DC_F32) {
            const bf16_t *pw = static_cast<const bf16_t *>(g.dc0) + (int64_t)batch * g.dc_batch_stride + (int64_t)(r0 + t * PK) * g.ldc + n0;
#pragma unroll
            for (int i = 0; i < WTileTr::NI; ++i)
                lds_dma<16>(pw, last ? offW_last[i] : offW[i], dst + P_ABYTES + (i * P_WAVES + wave) * 1024);
        }
    };
    // Rows past the end of the chunk re-read its last row; their copies in the tiles are replaced
    // by zeros, each lane clearing exactly the 16 bytes its own loads wrote (after waiting for them).
    auto clear_tail = [&](int slot) {
        if (tail == PK) return;
        char *dst = smem + slot * P_SLOT;
#pragma unroll
        for (int i = 0; i < WTileTr::NI; ++i) {
            const int row = (i * P_WAVES + wave) * 2 + lane / 32;
            if (row >= tail) {
                *reinterpret_cast<f32x4 *>(dst + (i * P_WAVES + wave) * 1024 + lane * 16) = f32x4{0.f, 0.f, 0.f, 0.f};
                if constexpr (!DC_F32)
                    *reinterpret_cast<f32x4 *>(dst + P_ABYTES + (i * P_WAVES + wave) * 1024 + lane * 16) = f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }
    };
    // float dC: thread `tid` converts the 8-column chunks tid, tid + 512, ... of the [64][256] tile
    // (chunk c is columns 8 (c % 32) .. + 7 of row c / 32) and writes them where the direct load would;
    // rows past the end of the chunk are written as zeros
    constexpr int FCH = PK * (PN / 8) / P_NT;       // chunks per thread
    f32x4 stage[DC_F32 ? 2 * FCH : 1];
    auto fetch_w = [&](int t) {
        if constexpr (DC_F32) {
            const int rows_here = t == T - 1 ? tail : PK;
#pragma unroll
            for (int i = 0; i < FCH; ++i) {
                const int c = i * P_NT + tid, row = min(c >> 5, rows_here - 1), col = min(c & 31, cols_n / 8 - 1);
                const int n = n0 + col * 8;
                const float *src = n < g.n_split ? static_cast<const float *>(g.dc0) + n : static_cast<const float *>(g.dc1) + (n - g.n_split);
                const f32x4 *p = reinterpret_cast<const f32x4 *>(src + (int64_t)batch * g.dc_batch_stride + (int64_t)(r0 + t * PK + row) * g.ldc);
                stage[2 * i] = p[0];
                stage[2 * i + 1] = p[1];
            }
        }
    };
    auto stash_w = [&](int t, int slot) {
        if constexpr (DC_F32) {
            const int rows_here = t == T - 1 ? tail : PK;
            char *dst = smem + slot * P_SLOT + P_ABYTES;
#pragma unroll
            for (int i = 0; i < FCH; ++i) {
                const int c = i * P_NT + tid, row = c >> 5, col = c & 31;
                bf16x8 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[e] = row < rows_here ? (bf16_t)stage[2 * i][e] : (bf16_t)0.f;
                    v[4 + e] = row < rows_here ? (bf16_t)stage[2 * i + 1][e] : (bf16_t)0.f;
                }
                *reinterpret_cast<bf16x8 *>(dst + row * (PN * 2) + ((col ^ (4 * (row & 3))) * 16)) = v;
            }
        }
    };

    int at_off[4], wt_off[2];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) at_off[mb] = WTileTr::lane_offset(lane, 4 * wm + mb);
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) wt_off[nb] = WTileTr::lane_offset(lane, 2 * wn + nb);

    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16 acc[4][2];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) acc[mb][nb] = zero16;

    struct Frags { Frag<bf16_t> fb[4], fw[2]; };
    auto load_frags = [&](const char *at, const char *wt, int ks, Frags &f) __attribute__((always_inline)) {
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) f.fw[nb] = WTileTr::load_frag(wt, ks, wt_off[nb]);
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) f.fb[mb] = WTileTr::load_frag(at, ks, at_off[mb]);
    };
    auto compute = [&](int slot) {
        const char *at = smem + slot * P_SLOT, *wt = at + P_ABYTES;
        Frags f[2];
        load_frags(at, wt, 0, f[0]);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if (ks + 1 < 4) load_frags(at, wt, ks + 1, f[(ks + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mb = 0; mb < 4; ++mb)
#pragma unroll
                for (int nb = 0; nb < 2; ++nb) acc[mb][nb] = mma(f[ks & 1].fw[nb], f[ks & 1].fb[mb], acc[mb][nb]);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // tile t is multiplied from slot t % 2 while tile t + 1 travels into the other slot; a float
    // dC tile is fetched into registers two tiles ahead and written to LDS one tile ahead
    fetch_w(0);
    issue(0, 0);
    stash_w(0, 0);
    if (T > 1) fetch_w(1);
    wait_vmem_all();
    if (T == 1) clear_tail(0);
    __syncthreads();
    for (int t = 0; t < T; ++t) {
        const int slot = t & 1;
        if (t + 1 < T) issue(t + 1, slot ^ 1);
        compute(slot);
        if (t + 1 < T) stash_w(t + 1, slot ^ 1);
        wait_vmem_all();
        if (t + 1 == T - 1) clear_tail(slot ^ 1);
        if (t + 2 < T) fetch_w(t + 2);
        __syncthreads();
    }

    // ---- the finished tile -> memory through LDS (whole rows written), 128 columns per pass; see
    // proj_gemm_kernel for the layout: element v of accumulator (mb, nb) is row 128 wm + 32 mb + lq,
    // column 64 wn + 32 nb + 8 (v / 4) + 4 hh + v % 4
    float *out = g.out + (int64_t)split * g.K * g.N + (int64_t)m0 * g.N + n0;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        if (pass) __syncthreads();
        if ((wn >> 1) == pass) {
#pragma unroll
            for (int mb = 0; mb < 4; ++mb) {
                const int m = 128 * wm + 32 * mb + lq;
                char *row = smem + m * 512;
#pragma unroll
                for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int c = 16 * (wn & 1) + 8 * nb + 2 * q + hh;
                        *reinterpret_cast<f32x4 *>(row + ((c ^ (m & 31)) * 16)) =
                            f32x4{acc[mb][nb][4 * q], acc[mb][nb][4 * q + 1], acc[mb][nb][4 * q + 2], acc[mb][nb][4 * q + 3]};
                    }
            }
        }
        __syncthreads();
        const int c = tid & 31;
        if (pass * 128 + c * 4 < cols_n) {
#pragma unroll
            for (int i = 0; i < PM / 16; ++i) {
                const int m = i * 16 + (tid >> 5);
                if (m < cols_m)
                    *reinterpret_cast<f32x4 *>(out + (int64_t)m * g.N + pass * 128 + c * 4) =
                        *reinterpret_cast<const f32x4 *>(smem + m * 512 + ((c ^ (m & 31)) * 16));
            }
        }
    }
}

template <bool A_ANY, bool W_TR, bool OUT_F32, int EPI = EPI_NONE>
hipError_t launch_proj(ProjArgs &args, int kernel_id, hipStream_t st)
{
    int wgs = 0;
    for (int j = 0; j < args.n_jobs; ++j) {
        ProjJob &J = args.job[j];
        J.m_tiles = (J.rows + PM - 1) / PM;
        J.n_tiles = (J.N + PN - 1) / PN;
        J.wg_begin = wgs;
        wgs += xcd_grid(J.batches * J.m_tiles, J.n_tiles);
    }
    if (wgs == 0) return hipSuccess;
    static std::once_flag once;
    static hipError_t attr = hipSuccess;
    std::call_once(once, [] {
        attr = hipFuncSetAttribute(reinterpret_cast<const void *>(proj_gemm_kernel<A_ANY, W_TR, OUT_F32, EPI>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, P_LDS);
    });
    if (attr != hipSuccess) return attr;
    TimedLaunch tl(kernel_id, st);
    hipLaunchKernelGGL((proj_gemm_kernel<A_ANY, W_TR, OUT_F32, EPI>), dim3(wgs), dim3(P_NT), P_LDS, st, args);
    return hipGetLastError();
}

} // namespace

hipError_t launch_project_qkv(const bf16_t *x, const bf16_t *w_q, const bf16_t *w_kv, int64_t s0, int l_s, int l_x,
                              int B, int E, bf16_t *q_seg, bf16_t *k, bf16_t *v, hipStream_t st)
{
    ProjArgs args{};
    args.lda = args.ldc = E;
    args.skip_tail = 0;
    int n = 0;
    {   // [K | V] = x [W_k | W_v]: the batches of x are contiguous, one tall matrix
        ProjJob &J = args.job[n++];
        J.a0 = x; J.a1 = nullptr; J.w = w_kv; J.c0 = k; J.c1 = v;
        J.a_batch_stride = J.c_batch_stride = 0;
        J.rows = J.rows_ok = B * l_x; J.batches = 1;
        J.N = 2 * E; J.K = E; J.k_split = E; J.n_split = E; J.ldw = 2 * E;
    }
    if (l_s > 0) {  // Q_i = x_i W_q
        ProjJob &J = args.job[n++];
        J.a0 = x + s0 * E; J.a1 = nullptr; J.w = w_q; J.c0 = q_seg; J.c1 = nullptr;
        J.a_batch_stride = (int64_t)l_x * E; J.c_batch_stride = (int64_t)l_s * E;
        J.rows = J.rows_ok = l_s; J.batches = B;
        J.N = E; J.K = E; J.k_split = E; J.n_split = E; J.ldw = E;
    }
    args.n_jobs = n;
    return launch_proj<false, true, false>(args, K_PROJ_FWD, st);
}

hipError_t launch_project_bwd(const bf16_t *dq, const float *dk_part, const float *dv_part, const bf16_t *w_q,
                              const bf16_t *w_kv, int l_s, int l_x, int rows_valid, int B, int E, int skip_tail,
                              float *dx_q, float *dx_part, hipStream_t st)
{
    ProjArgs args{};
    args.lda = args.ldc = E;
    args.skip_tail = skip_tail;
    int n = 0;
    {   // dx_partial = dK_part W_k^T + dV_part W_v^T: one contraction over the 2E columns of [dK | dV]
        ProjJob &J = args.job[n++];
        J.a0 = dk_part; J.a1 = dv_part; J.w = w_kv; J.c0 = dx_part; J.c1 = nullptr;
        J.a_batch_stride = J.c_batch_stride = (int64_t)l_x * E;
        J.rows = l_x; J.rows_ok = rows_valid; J.batches = B;
        J.N = E; J.K = 2 * E; J.k_split = E; J.n_split = E; J.ldw = 2 * E;
        J.a_f32 = 1;
    }
    if (l_s > 0) {  // dx_q = dQ_i W_q^T, in the same launch
        ProjJob &J = args.job[n++];
        J.a0 = dq; J.a1 = nullptr; J.w = w_q; J.c0 = dx_q; J.c1 = nullptr;
        J.a_batch_stride = J.c_batch_stride = (int64_t)l_s * E;
        J.rows = J.rows_ok = l_s; J.batches = B;
        J.N = E; J.K = E; J.k_split = E; J.n_split = E; J.ldw = E;
        J.a_f32 = 0;
    }
    args.n_jobs = n;
    return launch_proj<true, false, true>(args, K_PROJ_BWD, st);
}

// c = a w for any row count: one job, one tall matrix; with gelu_c also gelu_c = GeLU(c)
hipError_t launch_linear_fwd(const bf16_t *a, const bf16_t *w, int rows, int K, int N, bf16_t *c, bf16_t *gelu_c,
                             hipStream_t st)
{
    ProjArgs args{};
    args.lda = K; args.ldc = N; args.skip_tail = 0; args.n_jobs = 1;
    ProjJob &J = args.job[0];
    J.a0 = a; J.a1 = nullptr; J.w = w; J.c0 = c; J.c1 = gelu_c;
    J.a_batch_stride = J.c_batch_stride = 0;
    J.rows = J.rows_ok = rows; J.batches = 1;
    J.N = N; J.K = K; J.k_split = K; J.n_split = N; J.ldw = N;
    if (gelu_c) return launch_proj<false, true, false, EPI_GELU>(args, K_LINEAR_FWD, st);
    return launch_proj<false, true, false>(args, K_LINEAR_FWD, st);
}

// da = dc w^T: w as stored, [K][N], is the [output column][contraction index] layout read plainly;
// with gelu_u, da = (dc w^T) * GeLU'(gelu_u)
hipError_t launch_linear_bwd_input(const bf16_t *dc, const bf16_t *w, const bf16_t *gelu_u, int rows, int K, int N,
                                   bf16_t *da, hipStream_t st)
{
    ProjArgs args{};
    args.lda = N; args.ldc = K; args.skip_tail = 0; args.n_jobs = 1;
    ProjJob &J = args.job[0];
    J.a0 = dc; J.a1 = gelu_u; J.w = w; J.c0 = da; J.c1 = nullptr;
    J.a_batch_stride = J.c_batch_stride = 0;
    J.rows = J.rows_ok = rows; J.batches = 1;
    J.N = K; J.K = N; J.k_split = N; J.n_split = K; J.ldw = N;
    if (gelu_u) return launch_proj<false, false, false, EPI_GELU_BWD>(args, K_LINEAR_BWD, st);
    return launch_proj<false, false, false>(args, K_LINEAR_BWD, st);
}

// How the rows are split for the weight gradient: about two workgroups per compute unit, at least
// eight 64-row tiles per workgroup; a chunk never crosses batch entries.  Shape-only, deterministic.
static int wgrad_want(int batches, int K, int N)       // chunks per batch entry aimed at; never exceeded
{
    const int tiles = ((K + PM - 1) / PM) * ((N + PN - 1) / PN);
    const int want = ((512 + tiles - 1) / tiles + batches - 1) / batches;
    return want < 1 ? 1 : want;
}
static void wgrad_plan(int rows, int batches, int K, int N, int &splits_per_batch, int &chunk_rows)
{
    const int R = (rows + PK - 1) / PK;
    const int want = wgrad_want(batches, K, N);
    int chunk_tiles = (R + want - 1) / want;
    if (chunk_tiles < 8) chunk_tiles = R < 8 ? R : 8;
    if (chunk_tiles < 1) chunk_tiles = 1;
    splits_per_batch = (R + chunk_tiles - 1) / chunk_tiles;
    if (splits_per_batch < 1) splits_per_batch = 1;
    chunk_rows = chunk_tiles * PK;
}

static size_t wgrad_scratch_bytes(int rows, int batches, int K, int N)
{
    int spb, chunk_rows;
    wgrad_plan(rows, batches, K, N, spb, chunk_rows);
    return batches * spb > 1 ? (size_t)batches * spb * K * N * sizeof(float) : 0;
}

// g: operands, rows, batches, K, N, strides filled in; dw [K][N]; rows >= 1, batches >= 1
template <bool DC_F32>
static hipError_t launch_wgrad(WgradArgs &g, float *dw, float *scratch, hipStream_t st)
{
    wgrad_plan(g.rows, g.batches, g.K, g.N, g.splits_per_batch, g.chunk_rows);
    const int splits = g.batches * g.splits_per_batch;
    g.out = splits > 1 ? scratch : dw;
    g.m_tiles = (g.K + PM - 1) / PM;
    g.n_tiles = (g.N + PN - 1) / PN;
    static std::once_flag once;
    static hipError_t attr = hipSuccess;
    std::call_once(once, [] {
        attr = hipFuncSetAttribute(reinterpret_cast<const void *>(wgrad_gemm_kernel<DC_F32>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, P_LDS);
    });
    if (attr != hipSuccess) return attr;
    {
        TimedLaunch tl(K_LINEAR_WGRAD, st);
        hipLaunchKernelGGL(wgrad_gemm_kernel<DC_F32>, dim3(xcd_grid(splits, g.m_tiles * g.n_tiles)), dim3(P_NT), P_LDS, st, g);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (splits == 1) return hipSuccess;
    std::vector<const float *> parts(splits);
    for (int i = 0; i < splits; ++i) parts[i] = scratch + (size_t)i * g.K * g.N;
    return launch_reduce(parts.data(), splits, nullptr, g.K, 1, 1, g.N, dw, st);   // chunk 0 + chunk 1 + ..., in that order
}

size_t linear_bwd_weight_scratch_bytes(int rows, int K, int N) { return wgrad_scratch_bytes(rows, 1, K, N); }

// dw = a^T dc.  rows >= 1.
hipError_t launch_linear_bwd_weight(const bf16_t *a, const bf16_t *dc, int rows, int K, int N, float *dw, float *scratch,
                                    hipStream_t st)
{
    WgradArgs g{};
    g.a = a; g.dc0 = dc; g.dc1 = nullptr;
    g.rows = rows; g.batches = 1; g.K = K; g.N = N; g.n_split = N; g.lda = K; g.ldc = N;
    return launch_wgrad<false>(g, dw, scratch, st);
}

// enough for any rows_valid <= l_x: a plan never has more chunks per batch entry than wgrad_want()
size_t project_bwd_weight_scratch_bytes(int l_s, int l_x, int B, int E)
{
    (void)l_x;
    const size_t q = l_s > 0 ? wgrad_scratch_bytes(l_s, B, E, E) : 0;
    const size_t kv = (size_t)B * wgrad_want(B, E, 2 * E) * E * 2 * E * sizeof(float);
    return q > kv ? q : kv;
}
size_t project_bwd_weight_scratch_needed(int l_s, int rows_valid, int B, int E)
{
    const size_t q = l_s > 0 ? wgrad_scratch_bytes(l_s, B, E, E) : 0;
    const size_t kv = rows_valid > 0 ? wgrad_scratch_bytes(rows_valid, B, E, 2 * E) : 0;
    return q > kv ? q : kv;
}

// dw_q = sum_b x_i^T dQ_i (l_s >= 1) and dw_kv = sum_b x[:rows_valid]^T [dK_part | dV_part][:rows_valid] (rows_valid >= 1);
// either is skipped when its row count is 0 (the caller writes the zeros)
hipError_t launch_project_bwd_weight(const bf16_t *x, const bf16_t *dq, const float *dk_part, const float *dv_part, int64_t s0,
                                     int l_s, int l_x, int rows_valid, int B, int E, float *dw_q, float *dw_kv, float *scratch,
                                     hipStream_t st)
{
    if (l_s > 0) {
        WgradArgs g{};
        g.a = x + s0 * E; g.a_batch_stride = (int64_t)l_x * E; g.lda = E;
        g.dc0 = dq; g.dc1 = nullptr; g.dc_batch_stride = (int64_t)l_s * E; g.ldc = E;
        g.rows = l_s; g.batches = B; g.K = E; g.N = E; g.n_split = E;
        const hipError_t e = launch_wgrad<false>(g, dw_q, scratch, st);
        if (e != hipSuccess) return e;
    }
    if (rows_valid > 0) {
        WgradArgs g{};
        g.a = x; g.a_batch_stride = (int64_t)l_x * E; g.lda = E;
        g.dc0 = dk_part; g.dc1 = dv_part; g.dc_batch_stride = (int64_t)l_x * E; g.ldc = E;
        g.rows = rows_valid; g.batches = B; g.K = E; g.N = 2 * E; g.n_split = E;
        return launch_wgrad<true>(g, dw_kv, scratch, st);
    }
    return hipSuccess;
}

} // namespace lss
