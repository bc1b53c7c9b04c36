// Tuned bf16 backward of Eq. 2 (Section 3, Principle 3) for gfx950: the two matrix kernels of
// lss_bwd.hip (same mathematics, same operand roles) rebuilt around
//   * in the dQ kernel at d = 64, 64 query rows per wavefront, so each LDS fragment feeds two
//     matrix instructions;
//   * row-major LDS tiles read transposed with DS_READ_B64_TR_B16 where the contraction runs over
//     tile rows (K^T for dQ, Q^T and dO^T for dK and dV) -- no transposing stores;
//   * double-buffered, register-staged tile loads with one barrier per tile;
//   * D = rowsum(dO * out) computed inside the dQ kernel (no separate launch).
#include "lss_bf16.h"
#include "lss_kernels.h"

namespace lss {

// ------------------------------------------------------------------------------------------ dQ
template <int D>
struct DqBf16Cfg {
    static constexpr int NB = D == 64 ? 2 : 1;          // 32-row query blocks per wavefront
    static constexpr int WAVES = 4, RW = 32 * NB;
    static constexpr int BR = WAVES * RW, BC = 64, NT = 256;
    static constexpr int KP = D + 8;    // pitch of the K and V tiles (elements)
};

template <int D>
__global__ __launch_bounds__(256, 2) void bwd_dq_bf16_kernel(
    SegShape s, const bf16_t *__restrict__ q, const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
    const bf16_t *__restrict__ out, const bf16_t *__restrict__ dO, const float *__restrict__ lse,
    float *__restrict__ Dv, bf16_t *__restrict__ dq, float *__restrict__ dq_part, int n_splits)
{
    using C = DqBf16Cfg<D>;
    constexpr int NB = C::NB;
    __shared__ __attribute__((aligned(16))) bf16_t sK[2][C::BC * C::KP];
    __shared__ __attribute__((aligned(16))) bf16_t sV[2][C::BC * C::KP];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lq = lane & 31, hh = lane >> 5;
    const int bh = blockIdx.y, b = bh / s.H, h = bh % s.H, split = blockIdx.z;
    // query tiles are dispatched last-first: under the causal mask the last tiles see the most
    // keys, and starting the longest workgroups first shortens the tail of the launch
    const int r0 = (gridDim.x - 1 - blockIdx.x) * C::BR;
    const int rw0 = r0 + wave * C::RW;
    const int64_t ld = (int64_t)s.H * D;

    const int r_last = min(r0 + C::BR, s.l_s) - 1;
    const int kv_end = s.causal ? (int)min<int64_t>(s.l_x, s.s0 + r_last + 1) : s.l_x;
    const int n_tiles = (kv_end + C::BC - 1) / C::BC;
    const int per = (n_tiles + n_splits - 1) / n_splits;
    const int t_begin = split * per, t_end = min(n_tiles, t_begin + per);

    const bool wave_on = rw0 < s.l_s;
    const int64_t g_wave_last = s.s0 + min(rw0 + C::RW, s.l_s) - 1;

    int r[NB];
    bool row_ok[NB];
    float L2[NB], Dr[NB];
    Frag<bf16_t> qf[NB][D / 16], gf[NB][D / 16];
#pragma unroll
    for (int qb = 0; qb < NB; ++qb) {
        r[qb] = rw0 + qb * 32 + lq;
        row_ok[qb] = r[qb] < s.l_s;
        // rows past the segment re-read its last row (unconditional loads); they are never stored,
        // and lse = +inf makes their P and dS exactly 0
        const int rc = min(r[qb], s.l_s - 1);
        const int64_t off = ((int64_t)b * s.l_s + rc) * ld + (int64_t)h * D + hh * 8;
        float dsum = 0.f;
#pragma unroll
        for (int kb = 0; kb < D / 16; ++kb) {
            qf[qb][kb] = load_frag<bf16_t>(q + off + kb * 16);
            gf[qb][kb] = load_frag<bf16_t>(dO + off + kb * 16);
            const Frag<bf16_t> of = load_frag<bf16_t>(out + off + kb * 16);
#pragma unroll
            for (int e = 0; e < 8; ++e) dsum += (float)gf[qb][kb].v[e] * (float)of.v[e];
        }
        dsum += __shfl_xor(dsum, 32);
        Dr[qb] = dsum;
        const float lv = lse[(int64_t)bh * s.l_s + rc];
        L2[qb] = row_ok[qb] ? lv * kLog2e : INFINITY;
        if (row_ok[qb] && hh == 0 && split == 0) Dv[(int64_t)bh * s.l_s + r[qb]] = dsum;
    }
    const float c = kLog2e / sqrtf((float)D);

    f32x16 acc[NB][D / 32];
#pragma unroll
    for (int qb = 0; qb < NB; ++qb)
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[qb][db][e] = 0.f;

    const bf16_t *kbase = k + (int64_t)b * s.l_x * ld + (int64_t)h * D;
    const bf16_t *vbase = v + (int64_t)b * s.l_x * ld + (int64_t)h * D;
    const int tr_off = tr_lane_offset(lane, C::KP);

    TileStage<D, C::BC> stK, stV;
    if (t_begin < t_end) {
        const int j0 = t_begin * C::BC;
        stK.fetch(kbase + (int64_t)j0 * ld, ld, s.l_x - j0, tid);
        stV.fetch(vbase + (int64_t)j0 * ld, ld, s.l_x - j0, tid);
        stK.commit(sK[0], C::KP, tid);
        stV.commit(sV[0], C::KP, tid);
    }
    wait_vmem_all();
    __syncthreads();

    for (int t = t_begin; t < t_end; ++t) {
        const int cur = (t - t_begin) & 1;
        const int j0 = t * C::BC;
        const bool more = t + 1 < t_end;
        if (more) {
            const int j1 = j0 + C::BC;
            stK.fetch(kbase + (int64_t)j1 * ld, ld, s.l_x - j1, tid);
            stV.fetch(vbase + (int64_t)j1 * ld, ld, s.l_x - j1, tid);
        }

        if (wave_on && !(s.causal && j0 > g_wave_last)) {
            const bf16_t *tK = sK[cur], *tV = sV[cur];
            const bool tail = j0 + C::BC > s.l_x;
            const bool diag = s.causal && (j0 + C::BC - 1 > s.s0 + rw0);
#pragma unroll
            for (int kb2 = 0; kb2 < 2; ++kb2) {
                f32x16 sc[NB], dp[NB];
#pragma unroll
                for (int qb = 0; qb < NB; ++qb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) { sc[qb][e] = 0.f; dp[qb][e] = 0.f; }
#pragma unroll
                for (int kb = 0; kb < D / 16; ++kb) {
                    const Frag<bf16_t> ak = load_frag<bf16_t>(&tK[(kb2 * 32 + lq) * C::KP + kb * 16 + hh * 8]);
                    const Frag<bf16_t> av = load_frag<bf16_t>(&tV[(kb2 * 32 + lq) * C::KP + kb * 16 + hh * 8]);
#pragma unroll
                    for (int qb = 0; qb < NB; ++qb) {
                        sc[qb] = mma(ak, qf[qb][kb], sc[qb]);
                        dp[qb] = mma(av, gf[qb][kb], dp[qb]);
                    }
                }
#pragma unroll
                for (int qb = 0; qb < NB; ++qb) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const float p = fast_exp2(sc[qb][e] * c - L2[qb]);
                        sc[qb][e] = p * (dp[qb][e] - Dr[qb]);
                    }
                    if (tail || diag) {
                        const int64_t last = s.causal ? min<int64_t>(s.s0 + r[qb], s.l_x - 1) : (int64_t)s.l_x - 1;
                        const int rel = (int)max<int64_t>(min<int64_t>(last - j0 - 4 * hh, 2 * C::BC), -1);
#pragma unroll
                        for (int e = 0; e < 16; ++e)
                            if (kb2 * 32 + 8 * (e >> 2) + (e & 3) > rel) sc[qb][e] = 0.f;
                    }
                }
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const int ks = kb2 * 2 + half;
                    Frag<bf16_t> df[NB];
#pragma unroll
                    for (int qb = 0; qb < NB; ++qb) df[qb] = acc_to_frag<bf16_t>(sc[qb], half);
#pragma unroll
                    for (int db = 0; db < D / 32; ++db) {
                        const Frag<bf16_t> a = load_frag_tr(tK, C::KP, ks * 16, db * 32, tr_off);
#pragma unroll
                        for (int qb = 0; qb < NB; ++qb) acc[qb][db] = mma(a, df[qb], acc[qb][db]);
                    }
                }
            }
        }

        if (more) {
            stK.commit(sK[cur ^ 1], C::KP, tid);
            stV.commit(sV[cur ^ 1], C::KP, tid);
        }
        __syncthreads();
    }

    const float scale = 1.f / sqrtf((float)D);
#pragma unroll
    for (int qb = 0; qb < NB; ++qb) {
        if (!row_ok[qb]) continue;
        if (n_splits == 1) {
            bf16_t *dst0 = dq + ((int64_t)b * s.l_s + r[qb]) * ld + (int64_t)h * D;
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4)
                    *reinterpret_cast<bf16x4 *>(dst0 + db * 32 + 8 * e4 + 4 * hh) =
                        pack4(acc[qb][db][4 * e4] * scale, acc[qb][db][4 * e4 + 1] * scale,
                              acc[qb][db][4 * e4 + 2] * scale, acc[qb][db][4 * e4 + 3] * scale);
        } else {
            float *dst0 = dq_part + (int64_t)split * s.B * s.l_s * ld + ((int64_t)b * s.l_s + r[qb]) * ld + (int64_t)h * D;
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4) {
                    f32x4 val;
#pragma unroll
                    for (int i = 0; i < 4; ++i) val[i] = acc[qb][db][4 * e4 + i] * scale;
                    *reinterpret_cast<f32x4 *>(dst0 + db * 32 + 8 * e4 + 4 * hh) = val;
                }
        }
    }
}

// ------------------------------------------------------------------------------------------ dK, dV
template <int D>
struct DkvBf16Cfg {
    // 32-row key blocks per wavefront.  One: two blocks would halve the LDS traffic per flop but
    // their accumulators leave room for only one wavefront per SIMD, which measures slower.
    static constexpr int NB = 1;
    static constexpr int WAVES = 4, KW = 32 * NB;       // key rows per wavefront
    static constexpr int BKV = WAVES * KW, BQ = 64, NT = 256;
    static constexpr int QP = D + 8;                    // pitch of the Q and dO tiles (elements)
};

template <int D>
__global__ __launch_bounds__(256, D == 64 ? 2 : 1) void bwd_dkv_bf16_kernel(
    SegShape s, const bf16_t *__restrict__ q, const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
    const bf16_t *__restrict__ dO, const float *__restrict__ lse, const float *__restrict__ Dv,
    float *__restrict__ dk_part, float *__restrict__ dv_part)
{
    using C = DkvBf16Cfg<D>;
    constexpr int NB = C::NB;
    __shared__ __attribute__((aligned(16))) bf16_t sQ[2][C::BQ * C::QP];
    __shared__ __attribute__((aligned(16))) bf16_t sG[2][C::BQ * C::QP];
    __shared__ __attribute__((aligned(16))) float sL[2][C::BQ];
    __shared__ __attribute__((aligned(16))) float sD[2][C::BQ];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lq = lane & 31, hh = lane >> 5;
    // grid: x = (batch, head), y = key tile.  Workgroups are dispatched x-fastest, so the tiles
    // with the longest query loops (lowest keys under the causal mask) start first and the tiles no
    // query sees (plain zero fill) come last; with B*H a multiple of 8 all tiles of one head also
    // land on one XCD and share its L2 copy of that head's Q and dO.
    const int bh = blockIdx.x, b = bh / s.H, h = bh % s.H;
    const int j0 = blockIdx.y * C::BKV;
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

    if (rq_begin >= s.l_s) {
        // no query of the segment sees this tile: its partial rows are zero (coalesced fill)
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

    int j[NB];
    bool key_ok[NB];
    Frag<bf16_t> kf[NB][D / 16], vf[NB][D / 16];
#pragma unroll
    for (int kb2 = 0; kb2 < NB; ++kb2) {
        j[kb2] = jw0 + kb2 * 32 + lq;
        key_ok[kb2] = j[kb2] < s.l_x;
        // keys past the sequence re-read its last row (unconditional loads); never stored
        const int64_t off = kv_base + (int64_t)min(j[kb2], s.l_x - 1) * ld + hh * 8;
#pragma unroll
        for (int kb = 0; kb < D / 16; ++kb) {
            kf[kb2][kb] = load_frag<bf16_t>(k + off + kb * 16);
            vf[kb2][kb] = load_frag<bf16_t>(v + off + kb * 16);
        }
    }

    f32x16 dk[NB][D / 32], dv[NB][D / 32];
#pragma unroll
    for (int kb2 = 0; kb2 < NB; ++kb2)
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) { dk[kb2][db][e] = 0.f; dv[kb2][db][e] = 0.f; }

    const float c = kLog2e / sqrtf((float)D);
    const bf16_t *qbase = q + (int64_t)b * s.l_s * ld + (int64_t)h * D;
    const bf16_t *gbase = dO + (int64_t)b * s.l_s * ld + (int64_t)h * D;
    const float *lbase = lse + (int64_t)bh * s.l_s, *dbase = Dv + (int64_t)bh * s.l_s;
    const int tr_off = tr_lane_offset(lane, C::QP);
    const bool wave_on = jw0 < s.l_x;

    TileStage<D, C::BQ> stQ, stG;
    float stL = 0.f, stD = 0.f;
    bool st_ok = false;
    auto fetch = [&](int rq0) {
        stQ.fetch(qbase + (int64_t)rq0 * ld, ld, s.l_s - rq0, tid);
        stG.fetch(gbase + (int64_t)rq0 * ld, ld, s.l_s - rq0, tid);
        // every thread loads (unconditionally, clamped); threads < BQ keep the value.  Nothing is
        // computed from the loaded values here, so that no memory wait lands before the tile's
        // matrix work.
        const int rr = rq0 + (tid & (C::BQ - 1));
        st_ok = rr < s.l_s;
        stL = lbase[min(rr, s.l_s - 1)];
        stD = dbase[min(rr, s.l_s - 1)];
    };
    auto commit = [&](int buf) {
        stQ.commit(sQ[buf], C::QP, tid);
        stG.commit(sG[buf], C::QP, tid);
        // rows past the segment: lse = +inf makes P (hence dS) exactly 0
        if (tid < C::BQ) { sL[buf][tid] = st_ok ? stL * kLog2e : INFINITY; sD[buf][tid] = st_ok ? stD : 0.f; }
    };
    fetch(rq_begin);
    commit(0);
    wait_vmem_all();
    __syncthreads();

    int it = 0;
    for (int rq0 = rq_begin; rq0 < s.l_s; rq0 += C::BQ, ++it) {
        const int cur = it & 1;
        const bool more = rq0 + C::BQ < s.l_s;
        if (more) fetch(rq0 + C::BQ);

        // skip if the wave has no keys, or every key of the wave lies after every row of the tile
        const int64_t g_tile_last = s.s0 + min(rq0 + C::BQ, s.l_s) - 1;
        if (wave_on && !(s.causal && jw0 > g_tile_last)) {
            const bf16_t *tQ = sQ[cur], *tG = sG[cur];
            const bool diag = s.causal && ((int64_t)jw0 + C::KW - 1 > s.s0 + rq0);
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                f32x16 sc[NB], dp[NB];
#pragma unroll
                for (int kb2 = 0; kb2 < NB; ++kb2)
#pragma unroll
                    for (int e = 0; e < 16; ++e) { sc[kb2][e] = 0.f; dp[kb2][e] = 0.f; }
#pragma unroll
                for (int kb = 0; kb < D / 16; ++kb) {
                    const Frag<bf16_t> aq = load_frag<bf16_t>(&tQ[(qb * 32 + lq) * C::QP + kb * 16 + hh * 8]);
                    const Frag<bf16_t> ag = load_frag<bf16_t>(&tG[(qb * 32 + lq) * C::QP + kb * 16 + hh * 8]);
#pragma unroll
                    for (int kb2 = 0; kb2 < NB; ++kb2) {
                        sc[kb2] = mma(aq, kf[kb2][kb], sc[kb2]);
                        dp[kb2] = mma(ag, vf[kb2][kb], dp[kb2]);
                    }
                }
                // C tile: column = this lane's key, element e = query row qb*32 + 8*(e/4) + 4*hh + e%4
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4) {
                    const int rl = qb * 32 + 8 * e4 + 4 * hh;
                    const f32x4 L4 = *reinterpret_cast<const f32x4 *>(&sL[cur][rl]);
                    const f32x4 D4 = *reinterpret_cast<const f32x4 *>(&sD[cur][rl]);
#pragma unroll
                    for (int kb2 = 0; kb2 < NB; ++kb2)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int e = 4 * e4 + i;
                            const float p = fast_exp2(sc[kb2][e] * c - L4[i]);
                            sc[kb2][e] = p;
                            dp[kb2][e] = p * (dp[kb2][e] - D4[i]);
                        }
                }
                if (diag) {
#pragma unroll
                    for (int kb2 = 0; kb2 < NB; ++kb2) {
                        // rows of this q-block that come before the lane's key are masked:
                        // row index within the block, 8*(e/4) + e%4 (+ 4*hh), below `first`
                        const int first = (int)max<int64_t>(min<int64_t>((int64_t)j[kb2] - s.s0 - rq0 - qb * 32 - 4 * hh, 64), 0);
#pragma unroll
                        for (int e = 0; e < 16; ++e)
                            if (8 * (e >> 2) + (e & 3) < first) { sc[kb2][e] = 0.f; dp[kb2][e] = 0.f; }
                    }
                }
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const int ks = qb * 2 + half;
                    Frag<bf16_t> pf[NB], df[NB];
#pragma unroll
                    for (int kb2 = 0; kb2 < NB; ++kb2) {
                        pf[kb2] = acc_to_frag<bf16_t>(sc[kb2], half);
                        df[kb2] = acc_to_frag<bf16_t>(dp[kb2], half);
                    }
#pragma unroll
                    for (int db = 0; db < D / 32; ++db) {
                        const Frag<bf16_t> agt = load_frag_tr(tG, C::QP, ks * 16, db * 32, tr_off);
                        const Frag<bf16_t> aqt = load_frag_tr(tQ, C::QP, ks * 16, db * 32, tr_off);
#pragma unroll
                        for (int kb2 = 0; kb2 < NB; ++kb2) {
                            dv[kb2][db] = mma(agt, pf[kb2], dv[kb2][db]);
                            dk[kb2][db] = mma(aqt, df[kb2], dk[kb2][db]);
                        }
                    }
                }
            }
        }

        if (more) commit(cur ^ 1);
        __syncthreads();
    }

    const float scale = 1.f / sqrtf((float)D);
#pragma unroll
    for (int kb2 = 0; kb2 < NB; ++kb2) {
        if (!key_ok[kb2]) continue;
        const int64_t off = kv_base + (int64_t)j[kb2] * ld;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                f32x4 a, bq;
#pragma unroll
                for (int i = 0; i < 4; ++i) { a[i] = dk[kb2][db][4 * e4 + i] * scale; bq[i] = dv[kb2][db][4 * e4 + i]; }
                const int col = db * 32 + 8 * e4 + 4 * hh;
                *reinterpret_cast<f32x4 *>(dk_part + off + col) = a;
                *reinterpret_cast<f32x4 *>(dv_part + off + col) = bq;
            }
    }
}

int dq_bf16_rows_per_workgroup(int d) { return d == 64 ? DqBf16Cfg<64>::BR : DqBf16Cfg<128>::BR; }

template <int D>
static hipError_t launch_bwd_bf16_d(const SegShape &s, const bf16_t *q, const bf16_t *k, const bf16_t *v,
                                    const bf16_t *out, const float *lse, const bf16_t *dO, bf16_t *dq,
                                    float *dk_part, float *dv_part, const Workspace &ws, int n_splits,
                                    hipStream_t st)
{
    hipError_t e;
    {
        using C = DqBf16Cfg<D>;
        dim3 grid((s.l_s + C::BR - 1) / C::BR, s.B * s.H, n_splits);
        TimedLaunch tl(K_DQ, st);
        hipLaunchKernelGGL((bwd_dq_bf16_kernel<D>), grid, dim3(C::NT), 0, st, s, q, k, v, out, dO, lse, ws.D, dq,
                           ws.dq_part, n_splits);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    {
        using C = DkvBf16Cfg<D>;
        dim3 grid(s.B * s.H, (s.l_x + C::BKV - 1) / C::BKV);
        TimedLaunch tl(K_DKV, st);
        hipLaunchKernelGGL((bwd_dkv_bf16_kernel<D>), grid, dim3(C::NT), 0, st, s, q, k, v, dO, lse, ws.D, dk_part,
                           dv_part);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    return hipSuccess;
}

// dQ kernel then dK/dV kernel; the caller runs the dQ split merge in between or after.
hipError_t launch_bwd_bf16_main(const SegShape &s, const bf16_t *q, const bf16_t *k, const bf16_t *v,
                                const bf16_t *out, const float *lse, const bf16_t *dO, bf16_t *dq, float *dk_part,
                                float *dv_part, const Workspace &ws, int n_splits, hipStream_t st)
{
    if (s.d == 64) return launch_bwd_bf16_d<64>(s, q, k, v, out, lse, dO, dq, dk_part, dv_part, ws, n_splits, st);
    return launch_bwd_bf16_d<128>(s, q, k, v, out, lse, dO, dq, dk_part, dv_part, ws, n_splits, st);
}

} // namespace lss
