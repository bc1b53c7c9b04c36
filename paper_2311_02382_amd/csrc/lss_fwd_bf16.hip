// Tuned bf16 forward of Eq. 2 (Section 3, Principle 3) for gfx950.
//
// Same mathematics and operand roles as the generic kernel in lss_fwd.hip (S^T = K Q^T with one
// query per lane, then O^T += V^T P^T with P^T fed straight from the S^T registers).  The keys are
// walked in blocks of 32 (two per 64-key K/V tile).  Per block g three stages:
//     A(g): S^T product (matrix),  B(g): weights P^T (vector: exp, row sum, bf16 packing),
//     C(g): O^T product (matrix).
// A wavefront issues in order, and vector work costs it several times the issue time of a matrix
// instruction, so the stages are software-pipelined: step g issues the matrix instructions of
// A(g+1) and C(g-1) with the vector work of B(g) spread between them.  K/V tiles travel
// global -> LDS directly (no registers in between), a full loop iteration ahead, into a ring of
// three unpadded, swizzled tiles; V is read transposed by DS_READ_B64_TR_B16.
//
// Softmax: B subtracts the running maximum m as it stands (no pass over the block first).  Only
// when the block's weights of some row add up to more than 2^8 -- so no weight can be larger
// without this being noticed: a score well above m, or a row seeing its first key -- does a rare,
// wavefront-uniform fix-up raise m to the exact maximum, rescale the row sum and the accumulator,
// and redo the block's weights.  The final division by the row sum, which uses the same m, makes
// the result independent of when m was raised.
#include "lss_bf16.h"
#include <type_traits>
#include "lss_kernels.h"

namespace lss {

template <int D>
struct FwdBf16Cfg {
    // d = 64: four wavefronts, up to three workgroups per compute unit.  d = 128: the K/V ring alone
    // takes 96 KB of LDS, so only one workgroup fits; it has eight wavefronts (two per SIMD, 256 query
    // rows sharing the tiles) so that one wavefront's vector work hides behind another's matrix work.
    static constexpr int WAVES = D == 64 ? 4 : 8, RW = 32;      // wavefronts; query rows per wavefront
    static constexpr int BR = WAVES * RW, BC = 64, NT = 64 * WAVES;
    static constexpr int RING = 3;                      // K/V tiles resident in LDS
    static constexpr int NU = D / 16;                   // operand steps of the S^T product; same for O^T
    using Tile = DirectTile<D, BC, WAVES>;
    static constexpr int OFF_V = Tile::BYTES, SLOT = 2 * Tile::BYTES;   // one ring slot: K tile, V tile
    static constexpr float kMaxBlockSum = 256.0f;       // 2^8: largest sum of a lane's weights of one block without a fix-up
};

// DROP: dropout on the weights (Section 2.2): the weight that multiplies V is dropped or scaled by
// 1 / (1 - p) according to drop_keep() of (seed, batch*head, global row, key); row sum and lse are
// those of the softmax.
template <int D, bool DROP>
__global__ __launch_bounds__(FwdBf16Cfg<D>::NT, D == 64 ? 2 : 1) void fwd_bf16_kernel(SegShape s, DropArgs dr, const bf16_t *__restrict__ q,
                                                                       const bf16_t *__restrict__ k,
                                                                       const bf16_t *__restrict__ v,
                                                                       bf16_t *__restrict__ out, float *__restrict__ lse,
                                                                       float *__restrict__ o_part,
                                                                       float *__restrict__ lse_part, int n_splits, int n_q_tiles)
{
    using C = FwdBf16Cfg<D>;
    using Tile = typename C::Tile;
    constexpr int NU = C::NU;
    // (dropout: behind the ring, the column keys of the last four tiles issued, 64 each)
    __shared__ __attribute__((aligned(1024))) char smem[C::RING * C::SLOT + (DROP ? 4 * C::BC * 4 : 0)];

    const int tid = threadIdx.x, lane = tid & 63, lq = lane & 31, hh = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // 1-D grid in XCD order (xcd_item): one head at a time per XCD, whose workgroups share its K and
    // V in that XCD's L2.  Within a head: query tiles, last first -- under the causal mask the last
    // tiles see the most keys, and starting the longest workgroups first shortens the tail of the
    // launch -- then key splits.
    const int bhs = s.B * s.H;
    int bh, inner;
    if (!xcd_item(blockIdx.x, bhs, n_q_tiles * n_splits, bh, inner)) return;
    const int b = bh / s.H, h = bh % s.H;
    const int q_tile = inner % n_q_tiles, split = inner / n_q_tiles;
    const int r0 = (n_q_tiles - 1 - q_tile) * C::BR;
    const int rw0 = r0 + wave * C::RW;                  // first row of this wavefront
    const int64_t ld = (int64_t)s.H * D;

    const int r_last = min(r0 + C::BR, s.l_s) - 1;
    const int kv_end = s.causal ? (int)min<int64_t>(s.l_x, s.s0 + r_last + 1) : s.l_x;
    const int n_tiles = (kv_end + C::BC - 1) / C::BC;
    const int per = (n_tiles + n_splits - 1) / n_splits;
    const int t_begin = split * per, t_end = min(n_tiles, t_begin + per);
    const int T = max(t_end - t_begin, 0);

    // this lane's query row (column of the S^T tile); rows past the segment re-read its last row
    // (unconditional loads), are computed like any other and never stored
    const int r = rw0 + lq;
    const bool row_ok = r < s.l_s;
    Frag<bf16_t> qf[NU];
    {
        const bf16_t *qp = q + ((int64_t)b * s.l_s + min(r, s.l_s - 1)) * ld + (int64_t)h * D + hh * 8;
#pragma unroll
        for (int kb = 0; kb < NU; ++kb) qf[kb] = load_frag<bf16_t>(qp + kb * 16);
    }
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16 o[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db) o[db] = zero16;
    float m = -INFINITY, l = 0.f;                       // running maximum (log2 domain); this lane's half of the row sum
    const float c = kLog2e / sqrtf((float)D);

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
        auto load_a = [&](const char *tile, int kb2, int kb, Frag<bf16_t> &fk) __attribute__((always_inline)) {
            fk = load_frag<bf16_t>(reinterpret_cast<const bf16_t *>(tile + kb2 * 32 * (D * 2) + a_off[kb]));
        };
        auto load_c = [&](const char *tile, int kb2, int u, Frag<bf16_t> &fv) __attribute__((always_inline)) {
            const int half = u / (D / 32), db = u % (D / 32);
            fv = load_frag_tr_sw<D>(tile + C::OFF_V, (kb2 * 2 + half) * 16, t_off[db]);
        };
        // Where the causal diagonal or the end of the sequence crosses a block (first key jb), the
        // masked elements of its finished S^T accumulator are set to -inf, which B turns into weight
        // 0: keys after the lane's row, and keys past the sequence (whose loads re-read its last
        // row).  C-tile element e of this lane is key 8*(e/4) + 4*hh + e%4 of the block.
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
        // B for elements [e0, e1) (pairs): weight = 2^(c * S - m); the pair is added to the row sum
        // and rounded to bf16 into the operand fragment of C.
        // A row that has seen no key yet (m = -inf) subtracts a huge negative number instead, so that
        // any real score gives weight +inf and forces the fix-up, while masked scores still give 0.
        u32x4 ck4;      // dropout: the column keys of four consecutive elements, read when the first is due
        auto b_elems = [&](const f32x16 &sc, float m_sub, int jb, int e0, int e1, float &psum, Frag<bf16_t> (&pf)[2])
            __attribute__((always_inline)) {
#pragma unroll
            for (int e = e0; e < e1; e += 2) {
                const float p0 = fast_exp2(sc[e] * c - m_sub), p1 = fast_exp2(sc[e + 1] * c - m_sub);
                psum += p0;
                psum += p1;
                if (DROP) {     // element e of this lane is key jb + 8 (e / 4) + 4 hh + e % 4
                    if ((e & 3) == 0)
                        ck4 = *reinterpret_cast<const u32x4 *>(ck_ring + (((jb >> 6) & 3) * C::BC + (jb & 63) + 8 * (e >> 2) + 4 * hh) * 4);
                    pf[e >> 3].v[e & 7] = (bf16_t)(drop_keep(drop_rk, ck4[e & 3], dr.thr) ? p0 * dr.scale : 0.f);
                    pf[e >> 3].v[(e & 7) + 1] = (bf16_t)(drop_keep(drop_rk, ck4[(e & 3) + 1], dr.thr) ? p1 * dr.scale : 0.f);
                } else {
                    pf[e >> 3].v[e & 7] = (bf16_t)p0; pf[e >> 3].v[(e & 7) + 1] = (bf16_t)p1;
                }
            }
        };
        auto m_sub_of = [](float mm) { return mm == -INFINITY ? -1e30f : mm; };
        // The fix-up: raise m to the exact maximum over what the row has seen including this block,
        // rescale what was accumulated under the old m (row sum l0 before this block; accumulator,
        // to which this block has not been added yet) and redo the block's weights.
        auto fixup = [&](const f32x16 &sc, int jb, float l0, Frag<bf16_t> (&pf)[2]) __attribute__((always_inline)) {
            float mx = -INFINITY;
#pragma unroll
            for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sc[e]);
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m, mx * c);
            const float alpha = (m == -INFINITY) ? 0.f : fast_exp2(m - m_new);
            m = m_new;
            l = l0 * alpha;
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) o[db][e] *= alpha;
            b_elems(sc, m_sub_of(m), jb, 0, 16, l, pf);
        };

        // One pipeline step.  A: block (tile_a, kb2_a) into sc_a.  B: sc_b, first key jb_b, packing
        // into pf_b.  C: block (tile_c, kb2_c) from pf_c into o.  Per unit the matrix instructions
        // go C, A (A, C in the last unit); after each one come the B elements that fall to its slot.  Operand fragments are
        // read from LDS one unit ahead of their use; those of the first unit by the step before
        // (ak[0], cv[0] on entry), and this step leaves there those of the next step: A on block
        // (tile_an, kb2_an), C on (tile_cn, kb2_cn).  `mid` runs before those last reads: the even
        // steps put the loop's barrier there, because the next step's blocks may lie in the tile
        // that the barrier publishes.
        Frag<bf16_t> ak[2], cv[2];
        auto step = [&](auto has_a, auto has_b, auto has_c, const char *tile_a, int kb2_a, f32x16 &sc_a, f32x16 &sc_b,
                        int jb_b, Frag<bf16_t> (&pf_b)[2], const char *tile_c, int kb2_c, Frag<bf16_t> (&pf_c)[2],
                        const char *tile_an, int kb2_an, const char *tile_cn, int kb2_cn, auto &&mid)
            __attribute__((always_inline)) {
            constexpr bool HA = decltype(has_a)::value, HB = decltype(has_b)::value, HC = decltype(has_c)::value;
            constexpr int NS = 2 * NU;                  // slots; 8 element pairs of B spread over them
            static_assert(NU % 2 == 0, "fragment double buffers assume an even number of units");
            const float l0 = l, m_sub = m_sub_of(m);
            auto b_slot = [&](int slot) __attribute__((always_inline)) {
                if (HB) {
                    const int e0 = 2 * (slot * 8 / NS), e1 = 2 * ((slot + 1) * 8 / NS);
                    __builtin_amdgcn_sched_barrier(0);
                    b_elems(sc_b, m_sub, jb_b, e0, e1, l, pf_b);
                    __builtin_amdgcn_sched_barrier(0);
                }
            };
            if (HB) {
                mask_s(jb_b, sc_b);
                // B's inputs pass through an empty asm here: its arithmetic depends on nothing else in
                // this step, and the compiler would otherwise move all of it out of the step, in one lump
                asm volatile("" : "+v"(sc_b));
            }
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                const int half = u / (D / 32), db = u % (D / 32);
                if (u + 1 < NU) {
                    if (HC) load_c(tile_c, kb2_c, u + 1, cv[(u + 1) & 1]);
                    if (HA) load_a(tile_a, kb2_a, u + 1, ak[(u + 1) & 1]);
                    __builtin_amdgcn_sched_barrier(0);
                    if (HC) o[db] = mma(cv[u & 1], pf_c[half], o[db]);
                    b_slot(2 * u);
                    if (HA) sc_a = mma(ak[u & 1], qf[u], u == 0 ? zero16 : sc_a);
                    b_slot(2 * u + 1);
                } else {
                    // last unit: A first, so that its result is there when the next step's B wants it
                    if (HA) sc_a = mma(ak[u & 1], qf[u], sc_a);
                    b_slot(2 * u);
                    mid();
                    load_c(tile_cn, kb2_cn, 0, cv[0]);
                    load_a(tile_an, kb2_an, 0, ak[0]);
                    __builtin_amdgcn_sched_barrier(0);
                    if (HC) o[db] = mma(cv[u & 1], pf_c[half], o[db]);
                    b_slot(2 * u + 1);
                }
            }
            if (HB) {
                // ... and its results through another one, so that it is not sunk below the step either
                asm volatile("" : "+v"(pf_b[0].v), "+v"(pf_b[1].v), "+v"(l));
                if (__any(!(l - l0 <= C::kMaxBlockSum))) fixup(sc_b, jb_b, l0, pf_b);
            }
        };
        using std::true_type;
        using std::false_type;

        // ---- pipeline.  Block g = keys (t_begin + g/2) * 64 + (g%2) * 32 ..; tile t = blocks 2t, 2t+1.
        issue_tile(t_begin, 0);
        if (T > 1) issue_tile(t_begin + 1, 1);
        wait_vmem_all();
        __syncthreads();

        if (rw0 >= s.l_s) {
            // None of this wavefront's rows exists (a partly filled last query tile): it only keeps moving
            // tiles and meeting the loop's barriers.
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

        f32x16 sc0, sc1;                                // even / odd blocks
        Frag<bf16_t> pf0[2], pf1[2];
        // step -1: A(0) alone.  The first loop step has no C(-1): it multiplies zeros with tile 0 instead.
        load_a(smem, 0, 0, ak[0]);
        auto nothing = [] {};
        step(true_type{}, false_type{}, false_type{}, smem, 0, sc0, sc1, 0, pf0, smem, 0, pf1, smem, 1, smem, 1, nothing);
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
            for (int e = 0; e < 8; ++e) pf1[half].v[e] = (bf16_t)0.f;

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
            step(true_type{}, true_type{}, true_type{}, t_cur, 1, sc1, sc0, j0, pf0, t > 0 ? t_prv : t_cur, 1, pf1, t_a2, 0,
                 t_cur, 0, [&] {
                     wait_vmem_all();
                     __syncthreads();
                     issue_ahead(t, prv);
                 });
            // odd step g = 2t+1: A(2t+2) [tile t+1, first half; past the end result unused], B(2t+1),
            // C(2t) [tile t, first half]
            step(true_type{}, true_type{}, true_type{}, t_a2, 0, sc0, sc1, j0 + 32, pf1, t_cur, 0, pf0, t_a2, 1, t_cur, 1,
                 nothing);
            cur = nxt;
        }
        // step 2T: C(2T-1) [tile T-1, second half] alone
        {
            const char *t_last = smem + (cur == 0 ? C::RING - 1 : cur - 1) * C::SLOT;
            step(false_type{}, false_type{}, true_type{}, smem, 0, sc0, sc0, 0, pf0, t_last, 1, pf1, smem, 0, t_last, 1, nothing);
        }
        wait_vmem_all();                                // the last, redundant prefetches must land before the workgroup's LDS is given away
    }

    const float l_tot = l + __shfl_xor(l, 32);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    const float lse_nat = l_tot > 0.f ? (m + log2f(l_tot)) * kLn2 : -INFINITY;
    if (!row_ok) return;
    if (n_splits == 1) {
        bf16_t *op = out + ((int64_t)b * s.l_s + r) * ld + (int64_t)h * D;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4)
                *reinterpret_cast<bf16x4 *>(op + db * 32 + 8 * e4 + 4 * hh) =
                    pack4(o[db][4 * e4] * inv, o[db][4 * e4 + 1] * inv, o[db][4 * e4 + 2] * inv, o[db][4 * e4 + 3] * inv);
        if (hh == 0) lse[(int64_t)bh * s.l_s + r] = lse_nat;
    } else {
        // a split's normalised output travels to the merge kernel in bf16 (half the bytes; the merged
        // row is rounded to bf16 anyway), its lse in fp32
        const int64_t row = ((int64_t)split * bhs + bh) * s.l_s + r;
        bf16_t *op = reinterpret_cast<bf16_t *>(o_part) + row * D;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4)
                *reinterpret_cast<bf16x4 *>(op + db * 32 + 8 * e4 + 4 * hh) =
                    pack4(o[db][4 * e4] * inv, o[db][4 * e4 + 1] * inv, o[db][4 * e4 + 2] * inv, o[db][4 * e4 + 3] * inv);
        if (hh == 0) lse_part[row] = lse_nat;
    }
}

int fwd_bf16_rows_per_workgroup(int d) { return d == 64 ? FwdBf16Cfg<64>::BR : FwdBf16Cfg<128>::BR; }

template <int D>
static hipError_t launch_fwd_main(const SegShape &s, const DropArgs &drop, const bf16_t *q, const bf16_t *k,
                                  const bf16_t *v, bf16_t *out, float *lse, const Workspace &ws, int n_splits, hipStream_t st)
{
    using C = FwdBf16Cfg<D>;
    const int n_q_tiles = (s.l_s + C::BR - 1) / C::BR;
    dim3 grid((unsigned)xcd_grid(s.B * s.H, n_q_tiles * n_splits));
    TimedLaunch tl(K_FWD_BF16, st);
    if (drop.thr != 0)
        hipLaunchKernelGGL((fwd_bf16_kernel<D, true>), grid, dim3(C::NT), 0, st, s, drop, q, k, v, out, lse, ws.o_part,
                           ws.lse_part, n_splits, n_q_tiles);
    else
        hipLaunchKernelGGL((fwd_bf16_kernel<D, false>), grid, dim3(C::NT), 0, st, s, drop, q, k, v, out, lse, ws.o_part,
                           ws.lse_part, n_splits, n_q_tiles);
    return hipGetLastError();
}

hipError_t launch_fwd_bf16_main(const SegShape &s, const DropArgs &drop, const bf16_t *q, const bf16_t *k,
                                const bf16_t *v, bf16_t *out, float *lse, const Workspace &ws, int n_splits, hipStream_t st)
{
    if (s.d == 64) return launch_fwd_main<64>(s, drop, q, k, v, out, lse, ws, n_splits, st);
    return launch_fwd_main<128>(s, drop, q, k, v, out, lse, ws, n_splits, st);
}

} // namespace lss
