// Tuned bf16 backward of Eq. 2 (Section 3, Principle 3) for gfx950: the two matrix kernels of
// lss_bwd.hip (same mathematics, same operand roles) rebuilt as two kinds of workgroup that share
// one launch (bwd_main_bf16_kernel):
//   * 32 x 32 blocks, three stages per block (score-side products, vector work, output-side
//     products), software-pipelined so that the vector work of one block sits between the matrix
//     instructions of its neighbours;
//   * 64-row tiles loaded global -> LDS directly into a ring of three unpadded, swizzled tiles, a
//     full loop iteration ahead, one barrier per tile;
//   * row-major LDS tiles read transposed with DS_READ_B64_TR_B16 where the contraction runs over
//     tile rows (K^T for dQ, Q^T and dO^T for dK and dV) -- no transposing stores;
//   * lse, D = rowsum(dO * out) and the masks folded into accumulator start values where the
//     layout allows (a small kernel prepares -D and -lse * sqrt(d) per row).
#include "lss_bf16.h"
#include <type_traits>
#include "lss_kernels.h"

namespace lss {

// ------------------------------------------------------------------------------------------ dQ
template <int D>
struct DqBf16Cfg {
    static constexpr int WAVES = 4, RW = 32;            // query rows per wavefront
    static constexpr int BR = WAVES * RW, BC = 64, NT = 256;
    static constexpr int RING = 3;                      // K/V tiles resident in LDS
    static constexpr int NU = D / 16;                   // operand steps of the S/dP products; same for dQ
    using Tile = DirectTile<D, BC>;
    static constexpr int OFF_V = Tile::BYTES, SLOT = 2 * Tile::BYTES;   // one ring slot: K tile, V tile
};

// Transposed formulation: S^T = K Q^T and dP^T = V dO^T put the wavefront's 32 queries on the lanes
// (lse and D are per-lane scalars), and dS^T comes out of the accumulators in the layout the
// dQ^T += K^T dS^T product wants as its second operand.  The keys are walked in blocks of 32 (two
// per 64-key K/V tile).  Per block g three stages:
//     A(g): S^T and dP^T products (matrix),  B(g): dS^T (vector: exp, multiplies, bf16 packing),
//     C(g): dQ^T product (matrix).
// As in the dK/dV kernel below the stages are software-pipelined, step g issuing the matrix
// instructions of A(g+1) and C(g-1) with the vector work of B(g) spread between them, over a ring
// of three K/V tiles that are loaded global -> LDS directly, a full loop iteration ahead.
// -D = -rowsum(dO * out) of the wavefront's rows comes from the preprocess kernel (`Dn`).
// DROP: dropout on the weights (mask M = keep / (1 - p), decided by drop_keep() of (seed,
// batch*head, global row, key)): dS = P * (M dP - D).
template <int D, bool DROP>
__device__ __forceinline__ void bwd_dq_body(char *smem, const SegShape &s, const DropArgs &dr, const bf16_t *__restrict__ q,
                                            const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
                                            const bf16_t *__restrict__ dO, const float *__restrict__ lse,
                                            const float *__restrict__ Dn, bf16_t *__restrict__ dq,
                                            float *__restrict__ dq_part, int n_splits, int q_tile, int n_q_tiles, int bh,
                                            int split)
{
    using C = DqBf16Cfg<D>;
    using Tile = typename C::Tile;
    constexpr int NU = C::NU;

    const int tid = threadIdx.x, lane = tid & 63, lq = lane & 31, hh = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int b = bh / s.H, h = bh % s.H;
    // query tiles are dispatched last-first: under the causal mask the last tiles see the most
    // keys, and starting the longest workgroups first shortens the tail of the launch
    const int r0 = (n_q_tiles - 1 - q_tile) * C::BR;
    const int rw0 = r0 + wave * C::RW;
    const int64_t ld = (int64_t)s.H * D;

    const int r_last = min(r0 + C::BR, s.l_s) - 1;
    const int kv_end = s.causal ? (int)min<int64_t>(s.l_x, s.s0 + r_last + 1) : s.l_x;
    const int n_tiles = (kv_end + C::BC - 1) / C::BC;
    const int per = (n_tiles + n_splits - 1) / n_splits;
    const int t_begin = split * per, t_end = min(n_tiles, t_begin + per);
    const int T = max(t_end - t_begin, 0);

    // this lane's query row (column of the S^T tile); rows past the segment re-read its last row
    // (unconditional loads), get lse = +inf, which makes their P and dS exactly 0, and are never stored
    const int r = rw0 + lq;
    const bool row_ok = r < s.l_s;
    Frag<bf16_t> qf[NU], gf[NU];
    float L2, Dr;
    {
        const int rc = min(r, s.l_s - 1);
        const int64_t off = ((int64_t)b * s.l_s + rc) * ld + (int64_t)h * D + hh * 8;
#pragma unroll
        for (int kb = 0; kb < NU; ++kb) {
            qf[kb] = load_frag<bf16_t>(q + off + kb * 16);
            gf[kb] = load_frag<bf16_t>(dO + off + kb * 16);
        }
        Dr = -Dn[(int64_t)bh * s.l_s + rc];
        const float lv = lse[(int64_t)bh * s.l_s + rc];
        L2 = row_ok ? lv * kLog2e : INFINITY;
    }
    const float c = kLog2e / sqrtf((float)D);
    // -D in all 16 accumulator slots: third operand of each block's first dP^T instruction
    f32x16 neg_d;
#pragma unroll
    for (int e = 0; e < 16; ++e) neg_d[e] = -Dr;
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    f32x16 acc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db) acc[db] = zero16;

    if (T > 0) {
        const bf16_t *kbase = k + (int64_t)b * s.l_x * ld + (int64_t)h * D;
        const bf16_t *vbase = v + (int64_t)b * s.l_x * ld + (int64_t)h * D;

        // dropout: this lane's row key; the column seed; the column keys of tile t (global tile index)
        // are computed once, by one wavefront when the tile's loads are issued, into quarter t % 4 of
        // a small ring behind the tiles -- published by the same barrier as the tile
        uint32_t drop_rk = 0u, drop_cs = 0u;
        if (DROP) { drop_rk = drop_row_key(dr.seed_lo, (uint32_t)bh, (uint32_t)(s.s0 + r)); drop_cs = drop_col_seed(dr.seed_hi); }
        char *const ck_ring = smem + C::RING * C::SLOT;

        // ---- tile loads, by all four wavefronts.  Branch-free on purpose: a branch inside a pipeline step
        // splits it into basic blocks, and the vector work that was meant to sit between the step's
        // matrix instructions is then moved behind the branch in one lump.
        uint32_t offF[Tile::NI], offD[Tile::NI];        // this lane's global offsets within a full tile; and what
        Tile::offsets(offF, ld, C::BC, wave, lane);     // must be added to them in the sequence's last, partial tile
        const int t_part = s.l_x % C::BC ? s.l_x / C::BC : -1;     // (rows past the end re-read the last row)
        {
            uint32_t offL[Tile::NI];
            Tile::offsets(offL, ld, t_part >= 0 ? s.l_x % C::BC : C::BC, wave, lane);
#pragma unroll
            for (int i = 0; i < Tile::NI; ++i) offD[i] = offL[i] - offF[i];
        }
        const uint32_t tile_bytes = (uint32_t)(C::BC * ld * 2);
        auto issue_tile = [&](int t, int slot) {
            const int j0 = t * C::BC;
            const uint32_t part = t == t_part ? ~0u : 0u;
            uint32_t off[Tile::NI];
#pragma unroll
            for (int i = 0; i < Tile::NI; ++i) off[i] = offF[i] + (offD[i] & part);
            static_assert(C::OFF_V == Tile::BYTES, "V tile follows K tile");
            Tile::issue_pair(tile_ptr(kbase, t, tile_bytes), tile_ptr(vbase, t, tile_bytes), off, smem + slot * C::SLOT, wave);
            if (DROP && wave == 0)
                reinterpret_cast<uint32_t *>(ck_ring)[(t & 3) * C::BC + lane] = drop_col_key(drop_cs, (uint32_t)(j0 + lane));
        };
        // the loop's prefetch: tile t + 2, or once more the last tile into a slot nobody reads any more
        auto issue_ahead = [&](int t, int slot) { issue_tile(t_begin + min(t + 2, T - 1), slot); };

        // ---- per-lane LDS offsets (bytes, within a tile)
        int a_off[NU];                                  // A-operand chunk of row lq for operand step kb
#pragma unroll
        for (int kb = 0; kb < NU; ++kb) a_off[kb] = Tile::chunk_offset(lq, 2 * kb + hh);
        int t_off[D / 32];                              // transposed reads, column block db
#pragma unroll
        for (int db = 0; db < D / 32; ++db) t_off[db] = tr_lane_offset_sw<D>(lane, db);

        // ---- stage pieces.  `tile` / `kb2` name a block: LDS address of its ring slot and which half of it.
        auto load_a = [&](const char *tile, int kb2, int kb, Frag<bf16_t> &fk, Frag<bf16_t> &fv) __attribute__((always_inline)) {
            const char *p = tile + kb2 * 32 * (D * 2) + a_off[kb];
            fk = load_frag<bf16_t>(reinterpret_cast<const bf16_t *>(p));
            fv = load_frag<bf16_t>(reinterpret_cast<const bf16_t *>(p + C::OFF_V));
        };
        auto load_c = [&](const char *tile, int kb2, int u, Frag<bf16_t> &fk) __attribute__((always_inline)) {
            const int half = u / (D / 32), db = u % (D / 32);
            fk = load_frag_tr_sw<D>(tile, (kb2 * 2 + half) * 16, t_off[db]);
        };
        // B for elements [e0, e1): P = 2^(c * S - lse * log2 e), dS = P * (dP - D); finished pairs are
        // rounded to bf16 into the operand fragments of C
        // An element's exponential and the multiply that consumes it are issued one element apart (the
        // multiply of element e - 1 follows the exponential of element e): a transcendental's result may not
        // be read by the very next instruction, and the slot that would otherwise idle is not free.
        u32x4 ck4;      // dropout: the column keys of four consecutive elements, read when the first is due
        auto b_elems = [&](f32x16 &sc, f32x16 &dp, int jb, int e0, int e1, Frag<bf16_t> (&df)[2]) __attribute__((always_inline)) {
            auto finish = [&](int i) __attribute__((always_inline)) {       // sc[i] holds P by now
                if (DROP) {     // dp holds dP - D; element i of this lane is key jb + 8 (i / 4) + 4 hh + i % 4
                    if ((i & 3) == 0)
                        ck4 = *reinterpret_cast<const u32x4 *>(ck_ring + (((jb >> 6) & 3) * C::BC + (jb & 63) + 8 * (i >> 2) + 4 * hh) * 4);
                    dp[i] = drop_keep(drop_rk, ck4[i & 3], dr.thr) ? (dp[i] + Dr) * dr.scale - Dr : -Dr;
                }
                dp[i] = sc[i] * dp[i];
                if (i & 1) { df[i >> 3].v[(i & 7) - 1] = (bf16_t)dp[i - 1]; df[i >> 3].v[i & 7] = (bf16_t)dp[i]; }
            };
#pragma unroll
            for (int e = e0; e < e1; ++e) {
                sc[e] = fast_exp2(sc[e] * c - L2);
                if (e > 0) finish(e - 1);
                if (e == 15) finish(15);
            }
        };
        // Where the causal diagonal or the end of the sequence crosses a block (first key jb), the
        // masked elements of its finished S^T accumulator are set to -inf before B, which turns them
        // into P = dS = 0: keys after the lane's row, and keys past the sequence (whose loads
        // re-read its last row).  C-tile element e of this lane is key 8*(e/4) + 4*hh + e%4 of the block.
        auto mask_s = [&](int jb, f32x16 &sc) __attribute__((always_inline)) {
            // (positions are below 2^30, checked on the host: 32-bit scalar compares, no vector work per step)
            const bool diag = s.causal && (jb + 31 > (int)s.s0 + rw0);
            if (diag || jb + 32 > s.l_x) {
                const int last = s.causal ? min((int)s.s0 + r, s.l_x - 1) : s.l_x - 1;
                const int rel = max(min(last - jb - 4 * hh, 64), -1);
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    if (8 * (e >> 2) + (e & 3) > rel) sc[e] = -INFINITY;
            }
        };

        // One pipeline step.  A: block (tile_a, kb2_a) into (sc_a, dp_a).  B: (sc_b, dp_b), first key
        // jb_b, packing into df_b.  C: block (tile_c, kb2_c) from df_c into acc.  Per unit the matrix
        // instructions go C, A, A (A, A, C in the last unit); after each one come the B elements that fall to its slot.
        // Operand fragments are read from LDS one unit ahead of their use; those of the first unit
        // by the step before (ak[0], av[0], ck[0] on entry), and this step leaves there those of
        // the next step: A on block (tile_an, kb2_an), C on (tile_cn, kb2_cn).  `mid` runs before
        // those last reads: the even steps put the loop's barrier there, because the next step's
        // blocks may lie in the tile that the barrier publishes.
        Frag<bf16_t> ak[2], av[2], ck[2];
        auto step = [&](auto has_a, auto has_b, auto has_c, const char *tile_a, int kb2_a, f32x16 &sc_a, f32x16 &dp_a,
                        f32x16 &sc_b, f32x16 &dp_b, int jb_b, Frag<bf16_t> (&df_b)[2], const char *tile_c, int kb2_c,
                        Frag<bf16_t> (&df_c)[2], const char *tile_an, int kb2_an, const char *tile_cn, int kb2_cn, auto &&mid)
            __attribute__((always_inline)) {
            constexpr bool HA = decltype(has_a)::value, HB = decltype(has_b)::value, HC = decltype(has_c)::value;
            constexpr int NS = 3 * NU;                  // slots; 16 elements of B spread over them
            static_assert(NU % 2 == 0, "fragment double buffers assume an even number of units");
            auto b_slot = [&](int slot) __attribute__((always_inline)) {
                if (HB) {
                    const int e0 = slot * 16 / NS, e1 = (slot + 1) * 16 / NS;
                    __builtin_amdgcn_sched_barrier(0);
                    b_elems(sc_b, dp_b, jb_b, e0, e1, df_b);
                    __builtin_amdgcn_sched_barrier(0);
                }
            };
            if (HB) {
                mask_s(jb_b, sc_b);
                // B's inputs pass through an empty asm here: its arithmetic depends on nothing else in
                // this step, and the compiler would otherwise move all of it out of the step, in one lump
                asm volatile("" : "+v"(sc_b), "+v"(dp_b));
            }
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                const int half = u / (D / 32), db = u % (D / 32);
                if (u + 1 < NU) {
                    if (HC) load_c(tile_c, kb2_c, u + 1, ck[(u + 1) & 1]);
                    if (HA) load_a(tile_a, kb2_a, u + 1, ak[(u + 1) & 1], av[(u + 1) & 1]);
                    __builtin_amdgcn_sched_barrier(0);
                    if (HC) acc[db] = mma(ck[u & 1], df_c[half], acc[db]);
                    b_slot(3 * u);
                    if (HA) sc_a = mma(ak[u & 1], qf[u], u == 0 ? zero16 : sc_a);
                    b_slot(3 * u + 1);
                    if (HA) dp_a = mma(av[u & 1], gf[u], u == 0 ? neg_d : dp_a);
                    b_slot(3 * u + 2);
                } else {
                    // last unit: A first, so that its results are there when the next step's B wants them
                    if (HA) sc_a = mma(ak[u & 1], qf[u], sc_a);
                    b_slot(3 * u);
                    if (HA) dp_a = mma(av[u & 1], gf[u], dp_a);
                    b_slot(3 * u + 1);
                    mid();
                    load_c(tile_cn, kb2_cn, 0, ck[0]);
                    load_a(tile_an, kb2_an, 0, ak[0], av[0]);
                    __builtin_amdgcn_sched_barrier(0);
                    if (HC) acc[db] = mma(ck[u & 1], df_c[half], acc[db]);
                    b_slot(3 * u + 2);
                }
            }
            // ... and its results through another one, so that it is not sunk below the step either
            if (HB) asm volatile("" : "+v"(df_b[0].v), "+v"(df_b[1].v));
        };
        using std::true_type;
        using std::false_type;

        // ---- pipeline.  Block g = keys (t_begin + g/2) * 64 + (g%2) * 32 ..; tile t = blocks 2t, 2t+1.
        issue_tile(t_begin, 0);
        if (T > 1) issue_tile(t_begin + 1, 1);
        wait_vmem_all();
        __syncthreads();

        if (rw0 >= s.l_s) {
            // None of this wavefront's rows exists (a partly filled last query tile; half the workgroup for
            // a segment of at most 64 rows): it only keeps moving tiles and meeting the loop's barriers.
            int cur = 0;
            for (int t = 0; t < T; ++t) {
                const int prv = cur == 0 ? C::RING - 1 : cur - 1;
                wait_vmem_all();
                __syncthreads();
                issue_ahead(t, prv);
                cur = cur == C::RING - 1 ? 0 : cur + 1;
            }
            wait_vmem_all();                            // the last, redundant prefetches must land before the workgroup's LDS is given away
            return;
        }

        f32x16 sc0, dp0, sc1, dp1;                      // even / odd blocks
        Frag<bf16_t> df0[2], df1[2];
        // step -1: A(0) alone.  The first loop step has no C(-1): it multiplies zeros with tile 0 instead.
        load_a(smem, 0, 0, ak[0], av[0]);
        auto nothing = [] {};
        step(true_type{}, false_type{}, false_type{}, smem, 0, sc0, dp0, sc1, dp1, 0, df0, smem, 0, df1, smem, 1, smem, 1, nothing);
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
            for (int e = 0; e < 8; ++e) df1[half].v[e] = (bf16_t)0.f;

        int cur = 0;                                    // ring slot of tile t
        for (int t = 0; t < T; ++t) {
            const int nxt = cur == C::RING - 1 ? 0 : cur + 1, prv = cur == 0 ? C::RING - 1 : cur - 1;
            const char *t_cur = smem + cur * C::SLOT, *t_nxt = smem + nxt * C::SLOT, *t_prv = smem + prv * C::SLOT;
            const char *t_a2 = t + 1 < T ? t_nxt : t_cur;   // tile of A(2t+2), A(2t+3); past the end: any resident tile
            const int j0 = (t_begin + t) * C::BC;
            // even step g = 2t: A(2t+1) [tile t, second half], B(2t), C(2t-1) [tile t-1, second half;
            // for t = 0 tile 0, times zero]
            // Before its last reads (which may touch tile t+1): tile t+1's loads, issued one iteration
            // ago, have landed for this wavefront; after the barrier for all, and every wavefront has
            // requested its last operands from tile t-1, whose slot takes tile t+2.
            step(true_type{}, true_type{}, true_type{}, t_cur, 1, sc1, dp1, sc0, dp0, j0, df0, t > 0 ? t_prv : t_cur, 1, df1,
                 t_a2, 0, t_cur, 0, [&] {
                     wait_vmem_all();
                     __syncthreads();
                     issue_ahead(t, prv);
                 });
            // odd step g = 2t+1: A(2t+2) [tile t+1, first half; past the end result unused], B(2t+1),
            // C(2t) [tile t, first half]
            step(true_type{}, true_type{}, true_type{}, t_a2, 0, sc0, dp0, sc1, dp1, j0 + 32, df1, t_cur, 0, df0, t_a2, 1, t_cur,
                 1, nothing);
            cur = nxt;
        }
        // step 2T: C(2T-1) [tile T-1, second half] alone
        {
            const char *t_last = smem + (cur == 0 ? C::RING - 1 : cur - 1) * C::SLOT;
            step(false_type{}, false_type{}, true_type{}, smem, 0, sc0, dp0, sc0, dp0, 0, df0, t_last, 1, df1, smem, 0, t_last,
                 1, nothing);
        }
        wait_vmem_all();                                // the last, redundant prefetches must land before the workgroup's LDS is given away
    }

    if (!row_ok) return;
    const float scale = 1.f / sqrtf((float)D);
    if (n_splits == 1) {
        bf16_t *dst0 = dq + ((int64_t)b * s.l_s + r) * ld + (int64_t)h * D;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4)
                *reinterpret_cast<bf16x4 *>(dst0 + db * 32 + 8 * e4 + 4 * hh) =
                    pack4(acc[db][4 * e4] * scale, acc[db][4 * e4 + 1] * scale, acc[db][4 * e4 + 2] * scale,
                          acc[db][4 * e4 + 3] * scale);
    } else {
        float *dst0 = dq_part + (int64_t)split * s.B * s.l_s * ld + ((int64_t)b * s.l_s + r) * ld + (int64_t)h * D;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                f32x4 val;
#pragma unroll
                for (int i = 0; i < 4; ++i) val[i] = acc[db][4 * e4 + i] * scale;
                *reinterpret_cast<f32x4 *>(dst0 + db * 32 + 8 * e4 + 4 * hh) = val;
            }
    }
}

// ------------------------------------------------------------------------------------------ dK, dV
// A wavefront's finished [32 keys][D] tile (accumulator layout: lane = key lq, element e of block db =
// column 32 db + 8 (e / 4) + 4 hh + e % 4) goes to memory through a wavefront-private LDS buffer of
// 32 * D * 4 bytes, so that every store instruction writes whole rows (1 KB contiguous per four or
// two keys) instead of 32-byte pieces of 32 rows.  16-byte chunk c of key row r sits at chunk
// position c ^ (r % chunks per row).  `rows_ok` keys of the block exist.
template <int D>
__device__ __forceinline__ void store_key_rows(char *buf, const f32x16 (&acc)[D / 32], float scale, float *__restrict__ dst,
                                               int64_t ld, int rows_ok, int lane)
{
    constexpr int CH = D / 4;                           // 16-byte chunks per row
    const int lq = lane & 31, hh = lane >> 5;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
            const int c = db * 8 + 2 * e4 + hh;
            *reinterpret_cast<f32x4 *>(buf + lq * (D * 4) + ((c ^ (lq & (CH - 1))) * 16)) =
                f32x4{acc[db][4 * e4] * scale, acc[db][4 * e4 + 1] * scale, acc[db][4 * e4 + 2] * scale, acc[db][4 * e4 + 3] * scale};
        }
    constexpr int RPI = 64 / CH;                        // rows per store instruction
#pragma unroll
    for (int i = 0; i < 32 / RPI; ++i) {
        const int row = i * RPI + lane / CH, c = lane % CH;
        const f32x4 val = *reinterpret_cast<const f32x4 *>(buf + row * (D * 4) + ((c ^ (row & (CH - 1))) * 16));
        if (row < rows_ok) *reinterpret_cast<f32x4 *>(dst + (int64_t)row * ld + c * 4) = val;
    }
}

template <int D, bool DROP = false>
struct DkvBf16Cfg {
    // One 32-row key block per wavefront.  Two blocks would halve the LDS traffic per flop but
    // their accumulators leave room for only one wavefront per SIMD, which measures slower.
    static constexpr int WAVES = 4, KW = 32;            // key rows per wavefront
    static constexpr int BKV = WAVES * KW, BQ = 64, NT = 256;
    static constexpr int RING = 3;                      // Q/dO tiles resident in LDS
    static constexpr int NU = D / 16;                   // operand steps of the S/dP products; same for dV/dK
    using Tile = DirectTile<D, BQ>;
    // one ring slot: Q tile, dO tile, 64 S-accumulator start values, 64 dP-accumulator start values
    // (with dropout also the 64 rows' generator keys)
    static constexpr int OFF_G = Tile::BYTES, OFF_L = 2 * Tile::BYTES, OFF_D = OFF_L + BQ * 4, OFF_R = OFF_D + BQ * 4;
    static constexpr int SLOT = OFF_R + (DROP ? BQ * 4 : 0);
};

// The query rows are walked in blocks of 32 (two per 64-row Q/dO tile).  Per block g three stages:
//     A(g): S and dP products (matrix),  B(g): weights P, dS (vector: exp, multiplies, bf16 packing),
//     C(g): dV^T and dK^T products (matrix).
// A wavefront issues in order, and vector work costs it several times the issue time of a matrix
// instruction, so the stages are software-pipelined: step g issues the matrix instructions of
// A(g+1) and C(g-1) with the vector work of B(g) spread between them, one element per matrix
// instruction.  Block g+1 may belong to the next tile and block g-1 to the previous one, hence a
// ring of three tiles in LDS; tiles travel global -> LDS directly, a full loop iteration ahead.
//
// With dropout (DROP) the weight that enters dV is A = P * M (M = 1 / (1 - p) where the weight is
// kept, else 0) and dS = A * dP - P * D; the dP accumulator still starts at -D, so with acc = dP - D
// this is dS = A * acc + (P - A) * (-D).  The keep decision of an element needs its row's key
// (precomputed per query row, travelling with the tile like the start values) and this lane's
// column key; -D of the element's row is read from the tile's start values a second time.
template <int D, bool DROP>
__device__ __forceinline__ void bwd_dkv_body(char *smem, const SegShape &s, const DropArgs &dr, const bf16_t *__restrict__ q,
                                             const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
                                             const bf16_t *__restrict__ dO, const float *__restrict__ Ls,
                                             const float *__restrict__ Dn, const uint32_t *__restrict__ row_key,
                                             float *__restrict__ dk_part, float *__restrict__ dv_part, int bh, int key_tile)
{
    using C = DkvBf16Cfg<D, DROP>;
    using Tile = typename C::Tile;
    constexpr int NU = C::NU;

    const int tid = threadIdx.x, lane = tid & 63, lq = lane & 31, hh = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int b = bh / s.H, h = bh % s.H;
    const int j0 = key_tile * C::BKV;
    const int jw0 = j0 + wave * C::KW;                  // first key of this wavefront
    const int64_t ld = (int64_t)s.H * D;
    const int64_t kv_base = (int64_t)b * s.l_x * ld + (int64_t)h * D;

    // first query row that sees any key of this workgroup's tile
    int rq_begin = 0;
    if (s.causal) {
        const int64_t first = (int64_t)j0 - s.s0;
        rq_begin = first > 0 ? (int)min<int64_t>(first, s.l_s) : 0;
        rq_begin = rq_begin / C::BQ * C::BQ;
    }

    if (s.causal && j0 >= s.s0 + s.l_s) {
        // no query of the segment sees this tile: its partial rows are zero (coalesced fill), or stay
        // unwritten if the caller asked for that
        if (s.skip_tail) return;
        constexpr int F4 = D / 4;                       // float4 per (row, head)
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
        for (int i = tid; i < C::BKV * F4; i += C::NT) {
            const int row = j0 + i / F4, c4 = (i % F4) * 4;
            if (row < s.l_x) {
                *reinterpret_cast<f32x4 *>(dk_part + kv_base + (int64_t)row * ld + c4) = z;
                *reinterpret_cast<f32x4 *>(dv_part + kv_base + (int64_t)row * ld + c4) = z;
            }
        }
        return;
    }

    // this lane's key (column of the S tile); keys past the sequence re-read its last row
    // (unconditional loads), take part in all the arithmetic and are never stored
    const int j = jw0 + lq;
    Frag<bf16_t> kf[NU], vf[NU];
    {
        const int64_t off = kv_base + (int64_t)min(j, s.l_x - 1) * ld + hh * 8;
#pragma unroll
        for (int kb = 0; kb < NU; ++kb) {
            kf[kb] = load_frag<bf16_t>(k + off + kb * 16);
            vf[kb] = load_frag<bf16_t>(v + off + kb * 16);
        }
    }
    if constexpr (D == 128) {
        // At d = 128 the kernel needs more than 256 registers and the allocator parks these 64 in the
        // accumulation half of the register file -- then copies each into a vector register before
        // every use (54 to 68 copies per 32 matrix instructions).  A matrix instruction can read its
        // B operand from that half directly: naming the class here makes it do so.
#pragma unroll
        for (int kb = 0; kb < NU; ++kb) {
            asm volatile("" : "+a"(kf[kb].v));
            asm volatile("" : "+a"(vf[kb].v));
        }
    }

    f32x16 dk[D / 32], dv[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) { dk[db][e] = 0.f; dv[db][e] = 0.f; }

    const float sqrt_d = sqrtf((float)D);
    const float c = kLog2e / sqrt_d;
    const bf16_t *qbase = q + (int64_t)b * s.l_s * ld + (int64_t)h * D;
    const bf16_t *gbase = dO + (int64_t)b * s.l_s * ld + (int64_t)h * D;
    const float *lbase = Ls + (int64_t)bh * s.l_s, *dbase = Dn + (int64_t)bh * s.l_s;
    const uint32_t *rbase = DROP ? row_key + (int64_t)bh * s.l_s : nullptr;
    const uint32_t drop_ck = DROP ? drop_col_key(drop_col_seed(dr.seed_hi), (uint32_t)j) : 0u;  // this lane's key

    // ---- tile loads: all four wavefronts move Q and dO, and the 64 start values of either kind (even
    // wavefronts -lse*sqrt(d), odd ones -D; each twice, which is cheaper than a branch inside a pipeline
    // step: a branch splits the step into basic blocks, and the vector work meant to sit between its
    // matrix instructions is then moved behind the branch in one lump)
    uint32_t offF[Tile::NI], offD[Tile::NI];            // this lane's global offsets within a full tile; and what
    Tile::offsets(offF, ld, C::BQ, wave, lane);         // must be added to them in the segment's last, partial tile
    const int tq_part = s.l_s % C::BQ ? s.l_s / C::BQ : -1;        // (rows past the end re-read the last row)
    {
        uint32_t offL[Tile::NI];
        Tile::offsets(offL, ld, tq_part >= 0 ? s.l_s % C::BQ : C::BQ, wave, lane);
#pragma unroll
        for (int i = 0; i < Tile::NI; ++i) offD[i] = offL[i] - offF[i];
    }
    const uint32_t tile_bytes = (uint32_t)(C::BQ * ld * 2);
    const float *const sv_base = (wave & 1) ? dbase : lbase;
    const int sv_off = (wave & 1) ? C::OFF_D : C::OFF_L;
    auto issue_tile = [&](int tq, int slot) {           // tile tq = query rows [64 tq, 64 tq + 64) of the segment
        const int rq0 = tq * C::BQ;
        const uint32_t part = tq == tq_part ? ~0u : 0u;
        uint32_t off[Tile::NI];
#pragma unroll
        for (int i = 0; i < Tile::NI; ++i) off[i] = offF[i] + (offD[i] & part);
        static_assert(C::OFF_G == Tile::BYTES, "dO tile follows Q tile");
        char *dst = smem + slot * C::SLOT;
        Tile::issue_pair(tile_ptr(qbase, tq, tile_bytes), tile_ptr(gbase, tq, tile_bytes), off, dst, wave);
        const uint32_t ro = (uint32_t)min(lane, s.l_s - rq0 - 1) * 4u;
        lds_dma<4>(sv_base + rq0, ro, dst + sv_off);
        if (DROP && wave == 2) lds_dma<4>(rbase + rq0, ro, dst + C::OFF_R);
    };

    // ---- per-lane LDS offsets (bytes, within a tile)
    int a_off[NU];                                      // A-operand chunk of row lq for operand step kb
#pragma unroll
    for (int kb = 0; kb < NU; ++kb) a_off[kb] = Tile::chunk_offset(lq, 2 * kb + hh);
    int t_off[D / 32];                                  // transposed reads, column block db
#pragma unroll
    for (int db = 0; db < D / 32; ++db) t_off[db] = tr_lane_offset_sw<D>(lane, db);

    // ---- stage pieces.  `tile` / `qb` name a block: LDS address of its ring slot and which half of it.
    auto load_a = [&](const char *tile, int qb, int kb, Frag<bf16_t> &fq, Frag<bf16_t> &fg) __attribute__((always_inline)) {
        const char *p = tile + qb * 32 * (D * 2) + a_off[kb];
        fq = load_frag<bf16_t>(reinterpret_cast<const bf16_t *>(p));
        fg = load_frag<bf16_t>(reinterpret_cast<const bf16_t *>(p + C::OFF_G));
    };
    auto load_c = [&](const char *tile, int qb, int u, Frag<bf16_t> &fq, Frag<bf16_t> &fg) __attribute__((always_inline)) {
        const int half = u / (D / 32), db = u % (D / 32);
        fq = load_frag_tr_sw<D>(tile, (qb * 2 + half) * 16, t_off[db]);
        fg = load_frag_tr_sw<D>(tile + C::OFF_G, (qb * 2 + half) * 16, t_off[db]);
    };
    // Accumulators of A start at -lse*sqrt(d) and -D of their rows: C-tile element e of this lane is
    // query row 8*(e/4) + 4*hh + e%4 of the block.  init_load reads the values of element groups
    // [g0, g1) (4 elements each).
    auto init_load = [&](const char *tile, int qb, int g0, int g1, f32x16 &sc, f32x16 &dp) __attribute__((always_inline)) {
#pragma unroll
        for (int e4 = g0; e4 < g1; ++e4) {
            const f32x4 l4 = *reinterpret_cast<const f32x4 *>(tile + C::OFF_L + (qb * 32 + 8 * e4 + 4 * hh) * 4);
            const f32x4 d4 = *reinterpret_cast<const f32x4 *>(tile + C::OFF_D + (qb * 32 + 8 * e4 + 4 * hh) * 4);
#pragma unroll
            for (int i = 0; i < 4; ++i) { sc[4 * e4 + i] = l4[i]; dp[4 * e4 + i] = d4[i]; }
        }
    };
    // Where the causal diagonal or the end of the segment crosses the block (first row: local row
    // r0), the masked elements start at -inf instead, which B turns into P = dS = 0: rows before
    // the lane's key, and rows past the segment (whose loads re-read its last row).
    auto init_mask = [&](int r0, f32x16 &sc) __attribute__((always_inline)) {
        const bool diag = s.causal && (jw0 + C::KW - 1 > (int)s.s0 + r0);      // positions are below 2^30: 32-bit scalar compare
        if (diag || r0 + 32 > s.l_s) {
            const int first = diag ? max(min(j - (int)s.s0 - r0 - 4 * hh, 64), 0) : 0;
            const int end = min(s.l_s - r0, 32) - 4 * hh;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int rr = 8 * (e >> 2) + (e & 3);
                if (rr < first || rr >= end) sc[e] = -INFINITY;
            }
        }
    };
    // B for elements [e0, e1): P = 2^(c * (S - lse*sqrt(d))), dS = P * (dP - D); finished pairs are
    // rounded to bf16 into the operand fragments of C
    // (dropout: `tile_b`, `qb_b` name B's block; the row keys and -D of four elements are read when
    // the first of them is due)
    // (An element's exponential and the multiplies that consume it are issued one element apart, as in the dQ
    // workgroups: a transcendental's result may not be read by the very next instruction.)
    u32x4 rk4;
    f32x4 nd4;
    auto b_elems = [&](const char *tile_b, int qb_b, f32x16 &sc, f32x16 &dp, int e0, int e1, Frag<bf16_t> (&pf)[2],
                       Frag<bf16_t> (&df)[2]) __attribute__((always_inline)) {
        auto finish = [&](int i) __attribute__((always_inline)) {           // sc[i] holds P by now
            if constexpr (DROP) {
                if ((i & 3) == 0) {
                    rk4 = *reinterpret_cast<const u32x4 *>(tile_b + C::OFF_R + (qb_b * 32 + 8 * (i >> 2) + 4 * hh) * 4);
                    nd4 = *reinterpret_cast<const f32x4 *>(tile_b + C::OFF_D + (qb_b * 32 + 8 * (i >> 2) + 4 * hh) * 4);
                }
                const float p = sc[i];
                const float a = drop_keep(rk4[i & 3], drop_ck, dr.thr) ? p * dr.scale : 0.f;
                sc[i] = a;
                dp[i] = a * dp[i] + (p - a) * nd4[i & 3];
            } else {
                dp[i] = sc[i] * dp[i];
            }
            if (i & 1) {
                pf[i >> 3].v[(i & 7) - 1] = (bf16_t)sc[i - 1]; pf[i >> 3].v[i & 7] = (bf16_t)sc[i];
                df[i >> 3].v[(i & 7) - 1] = (bf16_t)dp[i - 1]; df[i >> 3].v[i & 7] = (bf16_t)dp[i];
            }
        };
#pragma unroll
        for (int e = e0; e < e1; ++e) {
            sc[e] = fast_exp2(sc[e] * c);
            if (e > 0) finish(e - 1);
            if (e == 15) finish(15);
        }
    };
    // One pipeline step.  A: block (tile_a, qb_a), first row r0_a, into (sc_a, dp_a).  B: (sc_b, dp_b),
    // packing into (pf_b, df_b).  C: block (tile_c, qb_c) from (pf_c, df_c) into dk, dv.  The matrix
    // instructions alternate C, C, A, A (A, A, C, C in the last unit); after each one come the B
    // elements that fall to its slot.
    // Everything read from LDS is requested well before its use: operand fragments one unit ahead;
    // for the next step (A on block (tile_an, qb_an), C on (tile_cn, qb_cn)) this step's last
    // unit requests the fragments of C's first unit (cq[0], cg[0]) and, into the three quarters of
    // B's registers that B is done with by then, the start values of A's accumulators (PRE says
    // the step before did that for this one).  `mid` runs before those last requests: the even
    // steps put the loop's barrier there, because the next step's A block may lie in the tile that
    // the barrier publishes.
    Frag<bf16_t> cq[2], cg[2];
    auto step = [&](auto has_a, auto has_b, auto has_c, auto pre, const char *tile_a, int qb_a, int r0_a, f32x16 &sc_a,
                    f32x16 &dp_a, const char *tile_b, int qb_b, f32x16 &sc_b, f32x16 &dp_b, Frag<bf16_t> (&pf_b)[2],
                    Frag<bf16_t> (&df_b)[2], const char *tile_c, int qb_c, Frag<bf16_t> (&pf_c)[2], Frag<bf16_t> (&df_c)[2],
                    const char *tile_an, int qb_an, const char *tile_cn, int qb_cn, auto &&mid) __attribute__((always_inline)) {
        constexpr bool HA = decltype(has_a)::value, HB = decltype(has_b)::value, HC = decltype(has_c)::value;
        constexpr bool PRE = decltype(pre)::value;
        constexpr int NS = 4 * NU;                      // slots; 16 elements of B spread over them
        static_assert(NU % 2 == 0, "fragment double buffers assume an even number of units");
        auto b_slot = [&](int slot) __attribute__((always_inline)) {
            if (HB) {
                const int e0 = slot * 16 / NS, e1 = (slot + 1) * 16 / NS;
                __builtin_amdgcn_sched_barrier(0);
                b_elems(tile_b, qb_b, sc_b, dp_b, e0, e1, pf_b, df_b);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        Frag<bf16_t> aq[2], ag[2];
        if (HA) {
            init_load(tile_a, qb_a, PRE ? 3 : 0, 4, sc_a, dp_a);
            load_a(tile_a, qb_a, 0, aq[0], ag[0]);
            init_mask(r0_a, sc_a);
        }
        // B's inputs pass through an empty asm here: its arithmetic depends on nothing else in this
        // step, and the compiler would otherwise move all of it out of the step, in one lump
        if (HB) asm volatile("" : "+v"(sc_b), "+v"(dp_b));
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const int half = u / (D / 32), db = u % (D / 32);
            if (u + 1 < NU) {
                if (HC) load_c(tile_c, qb_c, u + 1, cq[(u + 1) & 1], cg[(u + 1) & 1]);
                __builtin_amdgcn_sched_barrier(0);
                if (HC) dv[db] = mma(cg[u & 1], pf_c[half], dv[db]);
                b_slot(4 * u);
                if (HC) dk[db] = mma(cq[u & 1], df_c[half], dk[db]);
                b_slot(4 * u + 1);
                if (HA) load_a(tile_a, qb_a, u + 1, aq[(u + 1) & 1], ag[(u + 1) & 1]);
                __builtin_amdgcn_sched_barrier(0);
                if (HA) sc_a = mma(aq[u & 1], kf[u], sc_a);
                b_slot(4 * u + 2);
                if (HA) dp_a = mma(ag[u & 1], vf[u], dp_a);
                b_slot(4 * u + 3);
            } else {
                // last unit: A first, so that its results are there when the next step's B wants them
                if (HA) sc_a = mma(aq[u & 1], kf[u], sc_a);
                b_slot(4 * u);
                if (HA) dp_a = mma(ag[u & 1], vf[u], dp_a);
                b_slot(4 * u + 1);
                mid();
                load_c(tile_cn, qb_cn, 0, cq[0], cg[0]);
                init_load(tile_an, qb_an, 0, 3, sc_b, dp_b);    // elements 0..11 of B are packed by now
                __builtin_amdgcn_sched_barrier(0);
                if (HC) dv[db] = mma(cg[u & 1], pf_c[half], dv[db]);
                b_slot(4 * u + 2);
                if (HC) dk[db] = mma(cq[u & 1], df_c[half], dk[db]);
                b_slot(4 * u + 3);
            }
        }
        // ... and its results through another one, so that it is not sunk below the step either
        if (HB) asm volatile("" : "+v"(pf_b[0].v), "+v"(pf_b[1].v), "+v"(df_b[0].v), "+v"(df_b[1].v));
    };
    using std::true_type;
    using std::false_type;

    // ---- pipeline.  Block g of this workgroup = rows rq_begin + 32 g ..; tile t = blocks 2t, 2t+1.
    const int T = (s.l_s - rq_begin + C::BQ - 1) / C::BQ, tq_begin = rq_begin / C::BQ;
    // the loop's prefetch: tile t + 2, or once more the last tile into a slot nobody reads any more
    auto issue_ahead = [&](int t, int slot) { issue_tile(tq_begin + min(t + 2, T - 1), slot); };
    issue_tile(tq_begin, 0);
    if (T > 1) issue_tile(tq_begin + 1, 1);
    wait_vmem_all();
    __syncthreads();

    f32x16 sc0, dp0, sc1, dp1;                          // even / odd blocks
    Frag<bf16_t> pf0[2], df0[2], pf1[2], df1[2];
    // step -1: A(0) alone (leaves the first loop step's C operands in cq[0], cg[0]).  That step has
    // no C(-1): it multiplies zeros with tile 0 instead.
    auto nothing = [] {};
    step(true_type{}, false_type{}, false_type{}, false_type{}, smem, 0, rq_begin, sc0, dp0, smem, 0, sc1, dp1, pf0, df0, smem, 0,
         pf1, df1, smem, 1, smem, 1, nothing);
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int e = 0; e < 8; ++e) { pf1[half].v[e] = (bf16_t)0.f; df1[half].v[e] = (bf16_t)0.f; }

    int cur = 0;                                        // ring slot of tile t
    for (int t = 0; t < T; ++t) {
        const int nxt = cur == C::RING - 1 ? 0 : cur + 1, prv = cur == 0 ? C::RING - 1 : cur - 1;
        const char *t_cur = smem + cur * C::SLOT, *t_nxt = smem + nxt * C::SLOT, *t_prv = smem + prv * C::SLOT;
        const char *t_a2 = t + 1 < T ? t_nxt : t_cur;   // tile of A(2t+2) and A(2t+3); past the end: any resident tile
        const int r0 = rq_begin + t * C::BQ;
        // even step g = 2t: A(2t+1) [tile t, second half], B(2t), C(2t-1) [tile t-1, second half;
        // for t = 0 tile 0, times zero]
        // Before its last requests (which may touch tile t+1): tile t+1's loads, issued one iteration
        // ago, have landed for this wavefront; after the barrier for all, and every wavefront has
        // requested its last operands from tile t-1, whose slot takes tile t+2.
        step(true_type{}, true_type{}, true_type{}, true_type{}, t_cur, 1, r0 + 32, sc1, dp1, t_cur, 0, sc0, dp0, pf0, df0,
             t > 0 ? t_prv : t_cur, 1, pf1, df1, t_a2, 0, t_cur, 0, [&] {
                 wait_vmem_all();
                 __syncthreads();
                 issue_ahead(t, prv);
             });
        // odd step g = 2t+1: A(2t+2) [tile t+1, first half; past the end result unused], B(2t+1),
        // C(2t) [tile t, first half]
        step(true_type{}, true_type{}, true_type{}, true_type{}, t_a2, 0, r0 + C::BQ, sc0, dp0, t_cur, 1, sc1, dp1, pf1, df1, t_cur,
             0, pf0, df0, t_a2, 1, t_cur, 1, nothing);
        cur = nxt;
    }
    // step 2T: C(2T-1) [tile T-1, second half] alone
    {
        const char *t_last = smem + (cur == 0 ? C::RING - 1 : cur - 1) * C::SLOT;
        step(false_type{}, false_type{}, true_type{}, false_type{}, smem, 0, 0, sc0, dp0, smem, 0, sc0, dp0, pf0, df0, t_last, 1, pf1,
             df1, smem, 0, t_last, 1, nothing);
    }

    // the ring is free once every wavefront has made its last reads and the last, redundant prefetches have landed
    wait_vmem_all();
    __syncthreads();
    {
        char *buf = smem + wave * (32 * D * 4);
        const int64_t off = kv_base + (int64_t)jw0 * ld;
        const int rows_ok = min(s.l_x - jw0, C::KW);
        store_key_rows<D>(buf, dk, 1.f / sqrt_d, dk_part + off, ld, rows_ok, lane);
        store_key_rows<D>(buf, dv, 1.f, dv_part + off, ld, rows_ok, lane);
    }
}

// dK/dV for a segment of at most 64 query rows (the segment length the paper's largest runs leave
// one GPU): every key tile then meets ONE Q/dO tile, and the pipeline above would spend most of its
// steps on its start and its end.  Here a workgroup loads that tile once and walks KT_PER_WG key tiles
// with it, one 32-key block per wavefront as above: both 32-row blocks' S and dP, then their weights,
// then dV^T and dK^T, in program order; the next key tile's K and V rows are requested from memory
// before the current one is computed.  After the first barrier the wavefronts never meet again.
constexpr int kSkinnyRows = 64, kSkinnyTilesPerWg = 4;
template <int D>
__device__ __forceinline__ void bwd_dkv_skinny_body(char *smem, const SegShape &s, const bf16_t *__restrict__ q,
                                                    const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
                                                    const bf16_t *__restrict__ dO, const float *__restrict__ Ls,
                                                    const float *__restrict__ Dn, float *__restrict__ dk_part,
                                                    float *__restrict__ dv_part, int bh, int tile_group)
{
    using C = DkvBf16Cfg<D>;
    using Tile = typename C::Tile;
    constexpr int NU = C::NU;
    static_assert(C::BQ == kSkinnyRows, "one Q/dO tile holds the whole segment");

    const int tid = threadIdx.x, lane = tid & 63, lq = lane & 31, hh = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int b = bh / s.H, h = bh % s.H;
    const int64_t ld = (int64_t)s.H * D;
    const int64_t kv_base = (int64_t)b * s.l_x * ld + (int64_t)h * D;
    const int n_key_tiles = (s.l_x + C::BKV - 1) / C::BKV;
    const int kt0 = tile_group * kSkinnyTilesPerWg, kt1 = min(kt0 + kSkinnyTilesPerWg, n_key_tiles);
    // key tiles from kt_vis on are seen by no query of the segment
    const int kt_vis = s.causal ? (int)min<int64_t>((s.s0 + s.l_s + C::BKV - 1) / C::BKV, n_key_tiles) : n_key_tiles;

    // ---- the segment's Q/dO tile and start values (slot 0), by all four wavefronts
    if (kt0 < kt_vis) {
        uint32_t off[Tile::NI];
        Tile::offsets(off, ld, s.l_s, wave, lane);
        const bf16_t *qbase = q + (int64_t)b * s.l_s * ld + (int64_t)h * D;
        const bf16_t *gbase = dO + (int64_t)b * s.l_s * ld + (int64_t)h * D;
        Tile::issue_pair(qbase, gbase, off, smem, wave);
        if (wave < 2) {
            const float *src = (wave == 0 ? Ls : Dn) + (int64_t)bh * s.l_s;
            lds_dma<4>(src, (uint32_t)min(lane, s.l_s - 1) * 4u, smem + (wave == 0 ? C::OFF_L : C::OFF_D));
        }
    }
    auto load_kv = [&](int kt, Frag<bf16_t> (&kf)[NU], Frag<bf16_t> (&vf)[NU]) __attribute__((always_inline)) {
        const int jj = kt * C::BKV + wave * C::KW + lq;
        const int64_t off = kv_base + (int64_t)min(jj, s.l_x - 1) * ld + hh * 8;
#pragma unroll
        for (int kb = 0; kb < NU; ++kb) {
            kf[kb] = load_frag<bf16_t>(k + off + kb * 16);
            vf[kb] = load_frag<bf16_t>(v + off + kb * 16);
        }
    };
    Frag<bf16_t> kf[NU], vf[NU], kf_n[NU], vf_n[NU];
    if (kt0 < kt_vis) load_kv(kt0, kf, vf);
    wait_vmem_all();
    __syncthreads();

    int a_off[NU], t_off[D / 32];
#pragma unroll
    for (int kb = 0; kb < NU; ++kb) a_off[kb] = Tile::chunk_offset(lq, 2 * kb + hh);
#pragma unroll
    for (int db = 0; db < D / 32; ++db) t_off[db] = tr_lane_offset_sw<D>(lane, db);
    const float sqrt_d = sqrtf((float)D);
    const float c = kLog2e / sqrt_d, scale = 1.f / sqrt_d;
    const int n_blocks = s.l_s > 32 ? 2 : 1;            // 32-row blocks that hold rows of the segment

    for (int kt = kt0; kt < kt1; ++kt) {
        const int j0 = kt * C::BKV;
        if (kt >= kt_vis) {
            // no query of the segment sees this tile: its partial rows are zero, or stay unwritten
            if (s.skip_tail) return;
            constexpr int F4 = D / 4;
            const f32x4 z = {0.f, 0.f, 0.f, 0.f};
            for (int i = tid; i < C::BKV * F4; i += C::NT) {
                const int row = j0 + i / F4, c4 = (i % F4) * 4;
                if (row < s.l_x) {
                    *reinterpret_cast<f32x4 *>(dk_part + kv_base + (int64_t)row * ld + c4) = z;
                    *reinterpret_cast<f32x4 *>(dv_part + kv_base + (int64_t)row * ld + c4) = z;
                }
            }
            continue;
        }
        const bool more = kt + 1 < kt1 && kt + 1 < kt_vis;
        if (more) load_kv(kt + 1, kf_n, vf_n);          // in flight while this tile is computed

        const int jw0 = j0 + wave * C::KW, j = jw0 + lq;
        f32x16 dk[D / 32], dv[D / 32];
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) { dk[db][e] = 0.f; dv[db][e] = 0.f; }
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            if (qb < n_blocks) {
                const int r0 = 32 * qb;
                // S and dP of the block, accumulators starting at -lse*sqrt(d) and -D of their rows (element
                // e of this lane is row 8*(e/4) + 4*hh + e%4), masked elements at -inf
                f32x16 sc, dp;
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4) {
                    const f32x4 l4 = *reinterpret_cast<const f32x4 *>(smem + C::OFF_L + (r0 + 8 * e4 + 4 * hh) * 4);
                    const f32x4 d4 = *reinterpret_cast<const f32x4 *>(smem + C::OFF_D + (r0 + 8 * e4 + 4 * hh) * 4);
#pragma unroll
                    for (int i = 0; i < 4; ++i) { sc[4 * e4 + i] = l4[i]; dp[4 * e4 + i] = d4[i]; }
                }
                {
                    const bool diag = s.causal && (jw0 + C::KW - 1 > (int)s.s0 + r0);
                    if (diag || r0 + 32 > s.l_s) {
                        const int first = diag ? max(min(j - (int)s.s0 - r0 - 4 * hh, 64), 0) : 0;
                        const int end = min(s.l_s - r0, 32) - 4 * hh;
#pragma unroll
                        for (int e = 0; e < 16; ++e) {
                            const int rr = 8 * (e >> 2) + (e & 3);
                            if (rr < first || rr >= end) sc[e] = -INFINITY;
                        }
                    }
                }
#pragma unroll
                for (int kb = 0; kb < NU; ++kb) {
                    const char *p = smem + r0 * (D * 2) + a_off[kb];
                    const Frag<bf16_t> fq = load_frag<bf16_t>(reinterpret_cast<const bf16_t *>(p));
                    const Frag<bf16_t> fg = load_frag<bf16_t>(reinterpret_cast<const bf16_t *>(p + C::OFF_G));
                    sc = mma(fq, kf[kb], sc);
                    dp = mma(fg, vf[kb], dp);
                }
                // weights: P = 2^(c * (S - lse*sqrt(d))), dS = P * (dP - D), rounded to bf16 operands
                Frag<bf16_t> pf[2], df[2];
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float pw = fast_exp2(sc[e] * c);
                    pf[e >> 3].v[e & 7] = (bf16_t)pw;
                    df[e >> 3].v[e & 7] = (bf16_t)(pw * dp[e]);
                }
                // dV^T += dO^T P, dK^T += Q^T dS
#pragma unroll
                for (int u = 0; u < NU; ++u) {
                    const int half = u / (D / 32), db = u % (D / 32);
                    const Frag<bf16_t> fq = load_frag_tr_sw<D>(smem, (qb * 2 + half) * 16, t_off[db]);
                    const Frag<bf16_t> fg = load_frag_tr_sw<D>(smem + C::OFF_G, (qb * 2 + half) * 16, t_off[db]);
                    dv[db] = mma(fg, pf[half], dv[db]);
                    dk[db] = mma(fq, df[half], dk[db]);
                }
            }
        }
        {   // (slots 1 and 2 of the ring are never used here: a staging buffer per wavefront)
            char *buf = smem + C::SLOT + wave * (32 * D * 4);
            const int64_t off = kv_base + (int64_t)jw0 * ld;
            const int rows_ok = min(s.l_x - jw0, C::KW);
            store_key_rows<D>(buf, dk, scale, dk_part + off, ld, rows_ok, lane);
            store_key_rows<D>(buf, dv, 1.f, dv_part + off, ld, rows_ok, lane);
        }
        if (more) {
#pragma unroll
            for (int kb = 0; kb < NU; ++kb) { kf[kb] = kf_n[kb]; vf[kb] = vf_n[kb]; }
        }
    }
}

int dq_bf16_rows_per_workgroup(int d) { return d == 64 ? DqBf16Cfg<64>::BR : DqBf16Cfg<128>::BR; }

// ------------------------------------------------------------------------------------------ launch
// Start values of the dK/dV accumulators, per query row: -D = -rowsum(dO * out) and -lse * sqrt(d).
// One 16-byte chunk of a row per thread, D/8 consecutive lanes per row.
// (dropout: also the generator's key of the row, for the dK/dV workgroups.)
template <int D, bool DROP>
__global__ __launch_bounds__(256) void bwd_prep_bf16_kernel(SegShape s, DropArgs dr, const bf16_t *__restrict__ out,
                                                            const bf16_t *__restrict__ dO, const float *__restrict__ lse,
                                                            float *__restrict__ Dn, float *__restrict__ Ls,
                                                            uint32_t *__restrict__ row_key)
{
    constexpr int CPR = D / 8;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t rows = (int64_t)s.B * s.l_s * s.H;
    const int64_t row = min(idx / CPR, rows - 1);       // memory order [b][r][h]; whole lane groups stay in range
    const int cpos = (int)(idx % CPR);
    const Frag<bf16_t> g = load_frag<bf16_t>(dO + row * D + cpos * 8);
    const Frag<bf16_t> o = load_frag<bf16_t>(out + row * D + cpos * 8);
    float dsum = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) dsum += (float)g.v[e] * (float)o.v[e];
#pragma unroll
    for (int sh = 1; sh < CPR; sh <<= 1) dsum += __shfl_xor(dsum, sh);
    if (cpos == 0 && idx / CPR < rows) {
        const int h = (int)(row % s.H), r = (int)((row / s.H) % s.l_s), b = (int)(row / ((int64_t)s.H * s.l_s));
        const int64_t o_idx = ((int64_t)b * s.H + h) * s.l_s + r;
        Dn[o_idx] = -dsum;
        Ls[o_idx] = -lse[o_idx] * sqrtf((float)D);
        if constexpr (DROP) row_key[o_idx] = drop_row_key(dr.seed_lo, (uint32_t)(b * s.H + h), (uint32_t)(s.s0 + r));
    }
}

// dQ and dK/dV in one launch: the two kinds of workgroup do not depend on each other, so together
// they fill the chip better than one after the other (each alone ends in a tail of part-filled
// compute units, and short segments are mostly tail).  Workgroups [0, n_dq) take the (batch*head,
// query tile, key split) triples of dQ -- with few key splits they are the longest of the launch
// and start first -- and the rest the (batch*head, key tile) pairs of dK/dV.  Both parts are laid
// out in XCD order (xcd_item): an XCD works on one head at a time, whose workgroups share that
// head's K, V, Q and dO in its L2; within a head the longest workgroups come first (last query
// tiles; first key tiles, the zero-fill ones last).
// SKINNY: segments of at most 64 rows, whose dK/dV workgroups take kSkinnyTilesPerWg key tiles each
// (n_key_tiles then counts those groups).
template <int D, bool DROP, bool SKINNY = false>
__global__ __launch_bounds__(256, D == 64 ? 2 : 1) void bwd_main_bf16_kernel(
    SegShape s, DropArgs dr, const bf16_t *__restrict__ q, const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
    const bf16_t *__restrict__ dO, const float *__restrict__ lse,
    const float *__restrict__ Ls, const float *__restrict__ Dn, const uint32_t *__restrict__ row_key, bf16_t *__restrict__ dq,
    float *__restrict__ dq_part, float *__restrict__ dk_part, float *__restrict__ dv_part, int n_splits, int n_dq, int n_q_tiles,
    int n_key_tiles)
{
    using DkvC = DkvBf16Cfg<D, DROP>;
    // (dropout: the dQ workgroups keep a ring of column keys, 4 x 64, behind their tiles)
    constexpr int SMEM_DQ = DqBf16Cfg<D>::RING * DqBf16Cfg<D>::SLOT + (DROP ? 4 * DqBf16Cfg<D>::BC * 4 : 0);
    constexpr int SMEM = SMEM_DQ > DkvC::RING * DkvC::SLOT ? SMEM_DQ : DkvC::RING * DkvC::SLOT;
    __shared__ __attribute__((aligned(1024))) char smem[SMEM];
    const int bhs = s.B * s.H;
    const int id = blockIdx.x;
    int bh, inner;
    if (id >= n_dq) {
        if (!xcd_item(id - n_dq, bhs, n_key_tiles, bh, inner)) return;
        if constexpr (SKINNY) bwd_dkv_skinny_body<D>(smem, s, q, k, v, dO, Ls, Dn, dk_part, dv_part, bh, inner);
        else bwd_dkv_body<D, DROP>(smem, s, dr, q, k, v, dO, Ls, Dn, row_key, dk_part, dv_part, bh, inner);
    } else {
        if (!xcd_item(id, bhs, n_q_tiles * n_splits, bh, inner)) return;
        bwd_dq_body<D, DROP>(smem, s, dr, q, k, v, dO, lse, Dn, dq, dq_part, n_splits, inner % n_q_tiles, n_q_tiles, bh,
                             inner / n_q_tiles);
    }
}

template <int D>
static hipError_t launch_bwd_bf16_d(const SegShape &s, const DropArgs &drop, const bf16_t *q, const bf16_t *k,
                                    const bf16_t *v, const bf16_t *out, const float *lse, const bf16_t *dO, bf16_t *dq,
                                    float *dk_part, float *dv_part, const Workspace &ws, int n_splits,
                                    hipStream_t st)
{
    hipError_t e;
    const bool with_drop = drop.thr != 0;
    {
        const int64_t items = (int64_t)s.B * s.l_s * s.H * (D / 8);
        const dim3 grid((unsigned)((items + 255) / 256));
        TimedLaunch tl(K_BWD_PREP_BF16, st);
        if (with_drop)
            hipLaunchKernelGGL((bwd_prep_bf16_kernel<D, true>), grid, dim3(256), 0, st, s, drop, out, dO, lse, ws.D, ws.Ls, ws.row_key);
        else
            hipLaunchKernelGGL((bwd_prep_bf16_kernel<D, false>), grid, dim3(256), 0, st, s, drop, out, dO, lse, ws.D, ws.Ls, ws.row_key);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    {
        const int n_q_tiles = (s.l_s + DqBf16Cfg<D>::BR - 1) / DqBf16Cfg<D>::BR;
        const bool skinny = !with_drop && s.l_s <= kSkinnyRows;
        int n_key_tiles = (s.l_x + DkvBf16Cfg<D>::BKV - 1) / DkvBf16Cfg<D>::BKV;
        if (skinny) n_key_tiles = (n_key_tiles + kSkinnyTilesPerWg - 1) / kSkinnyTilesPerWg;      // groups of key tiles
        const int n_dq = xcd_grid(s.B * s.H, n_q_tiles * n_splits), n_dkv = xcd_grid(s.B * s.H, n_key_tiles);
        const dim3 grid((unsigned)(n_dkv + n_dq));
        TimedLaunch tl(K_BWD_MAIN_BF16, st);
        if (skinny)
            hipLaunchKernelGGL((bwd_main_bf16_kernel<D, false, true>), grid, dim3(256), 0, st, s, drop, q, k, v, dO, lse, ws.Ls,
                               ws.D, ws.row_key, dq, ws.dq_part, dk_part, dv_part, n_splits, n_dq, n_q_tiles, n_key_tiles);
        else if (with_drop)
            hipLaunchKernelGGL((bwd_main_bf16_kernel<D, true>), grid, dim3(256), 0, st, s, drop, q, k, v, dO, lse, ws.Ls, ws.D,
                               ws.row_key, dq, ws.dq_part, dk_part, dv_part, n_splits, n_dq, n_q_tiles, n_key_tiles);
        else
            hipLaunchKernelGGL((bwd_main_bf16_kernel<D, false>), grid, dim3(256), 0, st, s, drop, q, k, v, dO, lse, ws.Ls, ws.D,
                               ws.row_key, dq, ws.dq_part, dk_part, dv_part, n_splits, n_dq, n_q_tiles, n_key_tiles);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    return hipSuccess;
}

// accumulator start values (with dropout also the rows' generator keys), then dQ and dK/dV in one
// launch; the caller runs the dQ split merge
hipError_t launch_bwd_bf16_main(const SegShape &s, const DropArgs &drop, const bf16_t *q, const bf16_t *k,
                                const bf16_t *v, const bf16_t *out, const float *lse, const bf16_t *dO, bf16_t *dq,
                                float *dk_part, float *dv_part, const Workspace &ws, int n_splits, hipStream_t st)
{
    if (s.d == 64) return launch_bwd_bf16_d<64>(s, drop, q, k, v, out, lse, dO, dq, dk_part, dv_part, ws, n_splits, st);
    return launch_bwd_bf16_d<128>(s, drop, q, k, v, out, lse, dO, dq, dk_part, dv_part, ws, n_splits, st);
}

} // namespace lss
