// Tuned bf16 forward of Eq. 2 (Section 3, Principle 3) for gfx950.
//
// Same mathematics and operand roles as the generic kernel in lss_fwd.hip (S^T = K Q^T with one
// query per lane, then O^T += V^T P^T with P^T fed straight from the S^T registers); what differs:
//   * a wavefront owns 64 query rows (two 32-column B blocks), so every K / V^T fragment read from
//     LDS feeds two matrix instructions -- LDS traffic per flop is halved;
//   * V stays row-major in LDS and is read transposed by DS_READ_B64_TR_B16 (no transposing store);
//   * K/V tiles are double-buffered: the next tile's global loads are in flight while the current
//     one is consumed, one barrier per tile;
//   * the running maximum is only raised when a score exceeds it by more than 2^8 (log2 domain), so
//     the accumulator rescale is a rare wave-uniform branch; weights stay <= 2^8 and the final
//     division by the row sum, which uses the same maximum, makes the result independent of it;
//   * waves whose rows are past the segment, or entirely above the causal diagonal for a tile, skip
//     that tile's arithmetic.
#include "lss_bf16.h"
#include "lss_kernels.h"

namespace lss {

// NB = 32-row query blocks per wavefront: 2 for d = 64; 1 for d = 128, where two blocks of
// accumulators do not fit the register file.
template <int D>
struct FwdBf16Cfg {
    static constexpr int NB = D == 64 ? 2 : 1;
    static constexpr int WAVES = 4, RW = 32 * NB;       // query rows per wavefront
    static constexpr int BR = WAVES * RW, BC = 64, NT = 256;
    static constexpr int KP = D + 8;                    // K tile pitch (elements): 16 rows hit 64 distinct banks
    static constexpr int VP = D + 8;                    // V tile pitch
    static constexpr float kRescaleThreshold = 8.0f;    // log2 domain
};

template <int D>
__global__ __launch_bounds__(256, 2) void fwd_bf16_kernel(SegShape s, const bf16_t *__restrict__ q,
                                                       const bf16_t *__restrict__ k,
                                                       const bf16_t *__restrict__ v, bf16_t *__restrict__ out,
                                                       float *__restrict__ lse, float *__restrict__ o_part,
                                                       float *__restrict__ lse_part, int n_splits)
{
    using C = FwdBf16Cfg<D>;
    constexpr int NB = C::NB;
    __shared__ __attribute__((aligned(16))) bf16_t sK[2][C::BC * C::KP];
    __shared__ __attribute__((aligned(16))) bf16_t sV[2][C::BC * C::VP];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lq = lane & 31, hh = lane >> 5;
    const int bh = blockIdx.y, b = bh / s.H, h = bh % s.H, split = blockIdx.z;
    // query tiles are dispatched last-first: under the causal mask the last tiles see the most
    // keys, and starting the longest workgroups first shortens the tail of the launch
    const int r0 = (gridDim.x - 1 - blockIdx.x) * C::BR;
    const int rw0 = r0 + wave * C::RW;                  // first row of this wavefront
    const int64_t ld = (int64_t)s.H * D;

    const int r_last = min(r0 + C::BR, s.l_s) - 1;
    const int kv_end = s.causal ? (int)min<int64_t>(s.l_x, s.s0 + r_last + 1) : s.l_x;
    const int n_tiles = (kv_end + C::BC - 1) / C::BC;
    const int per = (n_tiles + n_splits - 1) / n_splits;
    const int t_begin = split * per, t_end = min(n_tiles, t_begin + per);

    const bool wave_on = rw0 < s.l_s;
    const int64_t g_wave_last = s.s0 + min(rw0 + C::RW, s.l_s) - 1;   // last global position of the wave

    int r[NB];
    bool row_ok[NB];
    Frag<bf16_t> qf[NB][D / 16];
#pragma unroll
    for (int qb = 0; qb < NB; ++qb) {
        r[qb] = rw0 + qb * 32 + lq;
        row_ok[qb] = r[qb] < s.l_s;
        // rows past the segment re-read its last row (unconditional loads); they are never stored
        const bf16_t *qp = q + ((int64_t)b * s.l_s + min(r[qb], s.l_s - 1)) * ld + (int64_t)h * D + hh * 8;
#pragma unroll
        for (int kb = 0; kb < D / 16; ++kb) qf[qb][kb] = load_frag<bf16_t>(qp + kb * 16);
    }

    f32x16 o[NB][D / 32];
#pragma unroll
    for (int qb = 0; qb < NB; ++qb)
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[qb][db][e] = 0.f;
    float m[NB], l[NB];
#pragma unroll
    for (int qb = 0; qb < NB; ++qb) { m[qb] = -INFINITY; l[qb] = 0.f; }
    const float c = kLog2e / sqrtf((float)D);

    const bf16_t *kbase = k + (int64_t)b * s.l_x * ld + (int64_t)h * D;
    const bf16_t *vbase = v + (int64_t)b * s.l_x * ld + (int64_t)h * D;
    const int tr_off = tr_lane_offset(lane, C::VP);

    TileStage<D, C::BC> stK, stV;
    if (t_begin < t_end) {
        const int j0 = t_begin * C::BC;
        stK.fetch(kbase + (int64_t)j0 * ld, ld, s.l_x - j0, tid);
        stV.fetch(vbase + (int64_t)j0 * ld, ld, s.l_x - j0, tid);
        stK.commit(sK[0], C::KP, tid);
        stV.commit(sV[0], C::VP, tid);
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

        // a wave takes part in a tile if it has rows and at least one of them sees the tile
        if (wave_on && !(s.causal && j0 > g_wave_last)) {
            const bf16_t *tK = sK[cur], *tV = sV[cur];
            f32x16 sc[NB][2];
#pragma unroll
            for (int kb2 = 0; kb2 < 2; ++kb2) {
#pragma unroll
                for (int qb = 0; qb < NB; ++qb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) sc[qb][kb2][e] = 0.f;
#pragma unroll
                for (int kb = 0; kb < D / 16; ++kb) {
                    const Frag<bf16_t> a = load_frag<bf16_t>(&tK[(kb2 * 32 + lq) * C::KP + kb * 16 + hh * 8]);
#pragma unroll
                    for (int qb = 0; qb < NB; ++qb) sc[qb][kb2] = mma(a, qf[qb][kb], sc[qb][kb2]);
                }
            }

            const bool tail = j0 + C::BC > s.l_x;
            const bool diag = s.causal && (j0 + C::BC - 1 > s.s0 + rw0);
            if (tail || diag) {
#pragma unroll
                for (int qb = 0; qb < NB; ++qb) {
                    // last visible key of this lane's query, relative to the lane's first key of the tile
                    const int64_t last = s.causal ? min<int64_t>(s.s0 + r[qb], s.l_x - 1) : (int64_t)s.l_x - 1;
                    const int rel = (int)max<int64_t>(min<int64_t>(last - j0 - 4 * hh, 2 * C::BC), -1);
#pragma unroll
                    for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
                        for (int e = 0; e < 16; ++e)
                            if (kb2 * 32 + 8 * (e >> 2) + (e & 3) > rel) sc[qb][kb2][e] = -INFINITY;
                }
            }

            float cand[NB];
            bool raise = false;
#pragma unroll
            for (int qb = 0; qb < NB; ++qb) {
                float mx = -INFINITY;
#pragma unroll
                for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
                    for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sc[qb][kb2][e]);
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                cand[qb] = mx * c;
                raise |= cand[qb] > m[qb] + C::kRescaleThreshold;
            }
            if (__any(raise)) {
#pragma unroll
                for (int qb = 0; qb < NB; ++qb) {
                    const float m_new = fmaxf(m[qb], cand[qb]);
                    const float alpha = (m_new == -INFINITY) ? 1.f : fast_exp2(m[qb] - m_new);
                    m[qb] = m_new;
                    l[qb] *= alpha;
#pragma unroll
                    for (int db = 0; db < D / 32; ++db)
#pragma unroll
                        for (int e = 0; e < 16; ++e) o[qb][db][e] *= alpha;
                }
            }
#pragma unroll
            for (int qb = 0; qb < NB; ++qb) {
                const float m_eff = (m[qb] == -INFINITY) ? 0.f : m[qb];
                float psum = 0.f;
#pragma unroll
                for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const float p = fast_exp2(sc[qb][kb2][e] * c - m_eff);
                        sc[qb][kb2][e] = p;
                        psum += p;
                    }
                l[qb] += psum;
            }

#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                Frag<bf16_t> pf[NB];
#pragma unroll
                for (int qb = 0; qb < NB; ++qb) pf[qb] = acc_to_frag<bf16_t>(sc[qb][ks >> 1], ks & 1);
#pragma unroll
                for (int db = 0; db < D / 32; ++db) {
                    const Frag<bf16_t> a = load_frag_tr(tV, C::VP, ks * 16, db * 32, tr_off);
#pragma unroll
                    for (int qb = 0; qb < NB; ++qb) o[qb][db] = mma(a, pf[qb], o[qb][db]);
                }
            }
        }

        if (more) {
            stK.commit(sK[cur ^ 1], C::KP, tid);
            stV.commit(sV[cur ^ 1], C::VP, tid);
        }
        __syncthreads();
    }

#pragma unroll
    for (int qb = 0; qb < NB; ++qb) {
        const float l_tot = l[qb] + __shfl_xor(l[qb], 32);
        const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
        const float lse_nat = l_tot > 0.f ? (m[qb] + log2f(l_tot)) * kLn2 : -INFINITY;
        if (!row_ok[qb]) continue;
        if (n_splits == 1) {
            bf16_t *op = out + ((int64_t)b * s.l_s + r[qb]) * ld + (int64_t)h * D;
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4)
                    *reinterpret_cast<bf16x4 *>(op + db * 32 + 8 * e4 + 4 * hh) =
                        pack4(o[qb][db][4 * e4] * inv, o[qb][db][4 * e4 + 1] * inv, o[qb][db][4 * e4 + 2] * inv,
                              o[qb][db][4 * e4 + 3] * inv);
            if (hh == 0) lse[(int64_t)bh * s.l_s + r[qb]] = lse_nat;
        } else {
            const int64_t row = ((int64_t)split * gridDim.y + bh) * s.l_s + r[qb];
            float *op = o_part + row * D;
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4) {
                    f32x4 val;
#pragma unroll
                    for (int i = 0; i < 4; ++i) val[i] = o[qb][db][4 * e4 + i] * inv;
                    *reinterpret_cast<f32x4 *>(op + db * 32 + 8 * e4 + 4 * hh) = val;
                }
            if (hh == 0) lse_part[row] = lse_nat;
        }
    }
}

int fwd_bf16_rows_per_workgroup(int d) { return d == 64 ? FwdBf16Cfg<64>::BR : FwdBf16Cfg<128>::BR; }

template <int D>
static hipError_t launch_fwd_main(const SegShape &s, const bf16_t *q, const bf16_t *k, const bf16_t *v, bf16_t *out,
                                  float *lse, const Workspace &ws, int n_splits, hipStream_t st)
{
    using C = FwdBf16Cfg<D>;
    dim3 grid((s.l_s + C::BR - 1) / C::BR, s.B * s.H, n_splits);
    TimedLaunch tl(K_FWD, st);
    hipLaunchKernelGGL((fwd_bf16_kernel<D>), grid, dim3(C::NT), 0, st, s, q, k, v, out, lse, ws.o_part, ws.lse_part,
                       n_splits);
    return hipGetLastError();
}

hipError_t launch_fwd_bf16_main(const SegShape &s, const bf16_t *q, const bf16_t *k, const bf16_t *v, bf16_t *out,
                                float *lse, const Workspace &ws, int n_splits, hipStream_t st)
{
    if (s.d == 64) return launch_fwd_main<64>(s, q, k, v, out, lse, ws, n_splits, st);
    return launch_fwd_main<128>(s, q, k, v, out, lse, ws, n_splits, st);
}

} // namespace lss
