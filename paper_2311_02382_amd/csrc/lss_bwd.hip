// Backward of Eq. 2 (Section 3, Principle 3) for one segment.  With P the softmax weights
// recomputed from lse, dP = dO V^T and D[r] = dO[r] . out[r] (= sum_j P dP):
//     dS = P * (dP - D);   dQ = dS K / sqrt(d);   dK_part = dS^T Q / sqrt(d);   dV_part = P^T dO.
// With dropout on the weights (template flag DROP; mask M = keep / (1 - p), out = (P * M) V): dP is
// replaced by M * dP and dV_part = (P * M)^T dO; D = dO . out still equals sum_j P (M dP).
// dK_part/dV_part hold this segment's contribution only; their sum over segments is the
// arithmetic of the reduce-scatter of Fig. 2(v).
//
// Three kernels, no atomics:
//   bwd_rowdot_kernel  D = rowsum(dO * out)
//   bwd_dq_kernel      query-tile owned (same shape as the forward kernel, split over key
//                      ranges); per key tile S^T = K Q^T, dP^T = V dO^T, dQ^T += K^T dS^T.
//   bwd_dkv_kernel     key-tile owned; loops over the query tiles that see the tile:
//                      S = Q K^T, dP = dO V^T, dV^T += dO^T P, dK^T += Q^T dS.
#include "lss_common.h"
#include "lss_kernels.h"

#include <type_traits>

namespace lss {

// ---------------------------------------------------------------- D = rowsum(dO * out)
template <typename T, int D>
__global__ __launch_bounds__(256) void bwd_rowdot_kernel(SegShape s, const T *__restrict__ out,
                                                         const T *__restrict__ dO, float *__restrict__ Dv)
{
    // 16 lanes per (b, r, h) row, each D/16 consecutive elements
    constexpr int PER = D / 16;
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t row = gid >> 4;          // (b * l_s + r) * H + h
    const int sub = (int)(gid & 15);
    const int64_t rows = (int64_t)s.B * s.l_s * s.H;
    float acc = 0.f;
    if (row < rows) {
        const T *o = out + row * D + sub * PER, *g = dO + row * D + sub * PER;
#pragma unroll
        for (int i = 0; i < PER; ++i) acc += (float)o[i] * (float)g[i];
    }
    acc += __shfl_xor(acc, 8);
    acc += __shfl_xor(acc, 4);
    acc += __shfl_xor(acc, 2);
    acc += __shfl_xor(acc, 1);
    if (row < rows && sub == 0) {
        const int64_t h = row % s.H, br = row / s.H, r = br % s.l_s, b = br / s.l_s;
        Dv[(b * s.H + h) * s.l_s + r] = acc;
    }
}

// ---------------------------------------------------------------- dQ
template <typename T, int D>
struct DqCfg {
    static constexpr int BR = 128, BC = 64, NT = 256;
    static constexpr int E = Elems16<T>::n;
    static constexpr int KP = D + E;    // pitch of the row-major K and V tiles
    static constexpr int TP = BC + E;   // pitch of the transposed K tile
};

template <typename T, int D, bool DROP>
__global__ __launch_bounds__(256) void bwd_dq_kernel(SegShape s, DropArgs dr, const T *__restrict__ q,
                                                     const T *__restrict__ k, const T *__restrict__ v,
                                                     const T *__restrict__ dO, const float *__restrict__ lse,
                                                     const float *__restrict__ Dv, T *__restrict__ dq,
                                                     float *__restrict__ dq_part, int n_splits)
{
    using C = DqCfg<T, D>;
    __shared__ __attribute__((aligned(16))) T sK[C::BC * C::KP];
    __shared__ __attribute__((aligned(16))) T sV[C::BC * C::KP];
    __shared__ __attribute__((aligned(16))) T sKt[D * C::TP];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lq = lane & 31, hh = lane >> 5;
    const int bh = blockIdx.y, b = bh / s.H, h = bh % s.H, split = blockIdx.z;
    const int r0 = blockIdx.x * C::BR;
    const int r = r0 + wave * 32 + lq;
    const bool row_ok = r < s.l_s;
    const int64_t g = s.s0 + r;
    const int64_t ld = (int64_t)s.H * D;

    const int r_last = min(r0 + C::BR, s.l_s) - 1;
    const int kv_end = s.causal ? (int)min<int64_t>(s.l_x, s.s0 + r_last + 1) : s.l_x;
    const int n_tiles = (kv_end + C::BC - 1) / C::BC;
    const int per = (n_tiles + n_splits - 1) / n_splits;
    const int t_begin = split * per, t_end = min(n_tiles, t_begin + per);

    Frag<T> qf[D / 16], gf[D / 16];
    {
        const int64_t off = ((int64_t)b * s.l_s + r) * ld + (int64_t)h * D + hh * 8;
#pragma unroll
        for (int kb = 0; kb < D / 16; ++kb) {
            qf[kb] = row_ok ? load_frag<T>(q + off + kb * 16) : zero_frag<T>();
            gf[kb] = row_ok ? load_frag<T>(dO + off + kb * 16) : zero_frag<T>();
        }
    }
    // rows past the segment get lse = +inf, so their P and dS are exactly 0
    const float L2 = row_ok ? lse[(int64_t)bh * s.l_s + r] * kLog2e : INFINITY;
    const float Dr = row_ok ? Dv[(int64_t)bh * s.l_s + r] : 0.f;
    const float c = kLog2e / sqrtf((float)D);
    uint32_t drop_rk = 0u, drop_cs = 0u;
    if (DROP) { drop_rk = drop_row_key(dr.seed_lo, (uint32_t)bh, (uint32_t)g); drop_cs = drop_col_seed(dr.seed_hi); }

    f32x16 acc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[db][e] = 0.f;

    const T *kbase = k + (int64_t)b * s.l_x * ld + (int64_t)h * D;
    const T *vbase = v + (int64_t)b * s.l_x * ld + (int64_t)h * D;

    for (int t = t_begin; t < t_end; ++t) {
        const int j0 = t * C::BC;
        __syncthreads();
        load_tile<T, D, C::BC, C::NT, C::KP, C::TP, true, true>(kbase + (int64_t)j0 * ld, ld, s.l_x - j0, sK, sKt, tid);
        load_tile<T, D, C::BC, C::NT, C::KP, 0, true, false>(vbase + (int64_t)j0 * ld, ld, s.l_x - j0, sV, nullptr, tid);
        __syncthreads();

        const bool tail = j0 + C::BC > s.l_x;
        const bool diag = s.causal && (j0 + C::BC - 1 > s.s0 + r0 + wave * 32);
        f32x16 ds[2];
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2) {
            f32x16 sc, dp;
#pragma unroll
            for (int e = 0; e < 16; ++e) { sc[e] = 0.f; dp[e] = 0.f; }
#pragma unroll
            for (int kb = 0; kb < D / 16; ++kb) {
                const Frag<T> ak = load_frag<T>(&sK[(kb2 * 32 + lq) * C::KP + kb * 16 + hh * 8]);
                sc = mma(ak, qf[kb], sc);
                const Frag<T> av = load_frag<T>(&sV[(kb2 * 32 + lq) * C::KP + kb * 16 + hh * 8]);
                dp = mma(av, gf[kb], dp);
            }
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                float p = fast_exp2(sc[e] * c - L2);
                if (tail || diag) {
                    const int key = j0 + kb2 * 32 + 8 * (e >> 2) + 4 * hh + (e & 3);
                    if (key >= s.l_x || (s.causal && key > g)) p = 0.f;
                }
                float dpe = dp[e];
                if (DROP) {
                    const int key = j0 + kb2 * 32 + 8 * (e >> 2) + 4 * hh + (e & 3);
                    dpe = drop_keep(drop_rk, drop_col_key(drop_cs, (uint32_t)key), dr.thr) ? dpe * dr.scale : 0.f;
                }
                ds[kb2][e] = p * (dpe - Dr);
            }
        }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const Frag<T> df = acc_to_frag<T>(ds[ks >> 1], ks & 1);
#pragma unroll
            for (int db = 0; db < D / 32; ++db) {
                const Frag<T> a = load_frag<T>(&sKt[(db * 32 + lq) * C::TP + ks * 16 + hh * 8]);
                acc[db] = mma(a, df, acc[db]);
            }
        }
    }
    if (!row_ok) return;

    const float scale = 1.f / sqrtf((float)D);
    if (n_splits == 1) {
        T *dst0 = dq + ((int64_t)b * s.l_s + r) * ld + (int64_t)h * D;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                T *dst = dst0 + db * 32 + 8 * e4 + 4 * hh;
#pragma unroll
                for (int i = 0; i < 4; ++i) dst[i] = (T)(acc[db][4 * e4 + i] * scale);
            }
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

// dq = sum over splits, in split order.
template <typename T>
__global__ __launch_bounds__(256) void bwd_dq_merge_kernel(const float *__restrict__ dq_part, int n_splits,
                                                           int64_t n4, T *__restrict__ dq)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n4) return;
    f32x4 acc = *reinterpret_cast<const f32x4 *>(dq_part + i * 4);
    for (int sp = 1; sp < n_splits; ++sp) acc += *reinterpret_cast<const f32x4 *>(dq_part + (sp * n4 + i) * 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) dq[i * 4 + e] = (T)acc[e];
}

// ---------------------------------------------------------------- dK, dV partials
template <typename T, int D>
struct DkvCfg {
    static constexpr int BKV = 128, BQ = 64, NT = 256;
    static constexpr int E = Elems16<T>::n;
    static constexpr int QP = D + E;    // pitch of the row-major Q and dO tiles
    static constexpr int TP = BQ + E;   // pitch of their transposed copies
};

template <typename T, int D, bool DROP>
__global__ __launch_bounds__(256) void bwd_dkv_kernel(SegShape s, DropArgs dr, const T *__restrict__ q,
                                                      const T *__restrict__ k, const T *__restrict__ v,
                                                      const T *__restrict__ dO, const float *__restrict__ lse,
                                                      const float *__restrict__ Dv,
                                                      float *__restrict__ dk_part, float *__restrict__ dv_part)
{
    using C = DkvCfg<T, D>;
    __shared__ __attribute__((aligned(16))) T sQ[C::BQ * C::QP];
    __shared__ __attribute__((aligned(16))) T sG[C::BQ * C::QP];
    __shared__ __attribute__((aligned(16))) T sQt[D * C::TP];
    __shared__ __attribute__((aligned(16))) T sGt[D * C::TP];
    __shared__ __attribute__((aligned(16))) float sL[C::BQ];
    __shared__ __attribute__((aligned(16))) float sD[C::BQ];
    __shared__ __attribute__((aligned(16))) uint32_t sRK[DROP ? C::BQ : 4];     // dropout: row keys of the tile's rows

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lq = lane & 31, hh = lane >> 5;
    const int bh = blockIdx.y, b = bh / s.H, h = bh % s.H;
    const int j0 = blockIdx.x * C::BKV;
    const int j = j0 + wave * 32 + lq;          // this lane's key row
    const bool key_ok = j < s.l_x;
    const int64_t ld = (int64_t)s.H * D;
    const int64_t kv_off = ((int64_t)b * s.l_x + j) * ld + (int64_t)h * D;

    const uint32_t drop_ck = DROP ? drop_col_key(drop_col_seed(dr.seed_hi), (uint32_t)j) : 0u;   // dropout: this lane's column key

    // first query row that sees any key of this tile
    int rq_begin = 0;
    if (s.causal) {
        const int64_t first = (int64_t)j0 - s.s0;
        rq_begin = first > 0 ? (int)min<int64_t>(first, s.l_s) : 0;
        rq_begin = rq_begin / C::BQ * C::BQ;
    }

    f32x16 dk[D / 32], dv[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) { dk[db][e] = 0.f; dv[db][e] = 0.f; }

    const bool hidden = s.causal && j0 >= s.s0 + s.l_s;     // no query of the segment sees this tile
    if (hidden && s.skip_tail) return;                      // the caller asked for such tiles to stay unwritten
    if (!hidden) {
        Frag<T> kf[D / 16], vf[D / 16];
#pragma unroll
        for (int kb = 0; kb < D / 16; ++kb) {
            kf[kb] = key_ok ? load_frag<T>(k + kv_off + kb * 16 + hh * 8) : zero_frag<T>();
            vf[kb] = key_ok ? load_frag<T>(v + kv_off + kb * 16 + hh * 8) : zero_frag<T>();
        }
        const float c = kLog2e / sqrtf((float)D);
        const T *qbase = q + (int64_t)b * s.l_s * ld + (int64_t)h * D;
        const T *gbase = dO + (int64_t)b * s.l_s * ld + (int64_t)h * D;

        for (int rq0 = rq_begin; rq0 < s.l_s; rq0 += C::BQ) {
            __syncthreads();
            load_tile<T, D, C::BQ, C::NT, C::QP, C::TP, true, true>(qbase + (int64_t)rq0 * ld, ld, s.l_s - rq0, sQ, sQt, tid);
            load_tile<T, D, C::BQ, C::NT, C::QP, C::TP, true, true>(gbase + (int64_t)rq0 * ld, ld, s.l_s - rq0, sG, sGt, tid);
            if (tid < C::BQ) {
                const int rr = rq0 + tid;
                // rows past the segment: lse = +inf makes P (hence dS) exactly 0
                sL[tid] = rr < s.l_s ? lse[(int64_t)bh * s.l_s + rr] * kLog2e : INFINITY;
                sD[tid] = rr < s.l_s ? Dv[(int64_t)bh * s.l_s + rr] : 0.f;
                if (DROP) sRK[tid] = drop_row_key(dr.seed_lo, (uint32_t)bh, (uint32_t)(s.s0 + rr));
            }
            __syncthreads();

            // does any (query, key) pair of this wavefront's 32 keys x 64 rows need the mask?
            const bool diag = s.causal && ((int64_t)j0 + wave * 32 + 31 > s.s0 + rq0);
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                f32x16 sc, dp;
#pragma unroll
                for (int e = 0; e < 16; ++e) { sc[e] = 0.f; dp[e] = 0.f; }
#pragma unroll
                for (int kb = 0; kb < D / 16; ++kb) {
                    const Frag<T> aq = load_frag<T>(&sQ[(qb * 32 + lq) * C::QP + kb * 16 + hh * 8]);
                    sc = mma(aq, kf[kb], sc);
                    const Frag<T> ag = load_frag<T>(&sG[(qb * 32 + lq) * C::QP + kb * 16 + hh * 8]);
                    dp = mma(ag, vf[kb], dp);
                }
                // C tile: column = this lane's key, element e = query row qb*32 + 8*(e/4) + 4*hh + e%4
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4) {
                    const int rl = qb * 32 + 8 * e4 + 4 * hh;
                    const f32x4 L4 = *reinterpret_cast<const f32x4 *>(&sL[rl]);
                    const f32x4 D4 = *reinterpret_cast<const f32x4 *>(&sD[rl]);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int e = 4 * e4 + i;
                        float p = fast_exp2(sc[e] * c - L4[i]);
                        if (diag && (int64_t)j > s.s0 + rq0 + rl + i) p = 0.f;
                        float pv = p, dpe = dp[e];
                        if (DROP) {
                            const float mk = drop_keep(sRK[rl + i], drop_ck, dr.thr) ? dr.scale : 0.f;
                            pv = p * mk;
                            dpe *= mk;
                        }
                        sc[e] = pv;
                        dp[e] = p * (dpe - D4[i]);
                    }
                }
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const int ks = qb * 2 + half;
                    const Frag<T> pf = acc_to_frag<T>(sc, half);
                    const Frag<T> df = acc_to_frag<T>(dp, half);
#pragma unroll
                    for (int db = 0; db < D / 32; ++db) {
                        const Frag<T> agt = load_frag<T>(&sGt[(db * 32 + lq) * C::TP + ks * 16 + hh * 8]);
                        dv[db] = mma(agt, pf, dv[db]);
                        const Frag<T> aqt = load_frag<T>(&sQt[(db * 32 + lq) * C::TP + ks * 16 + hh * 8]);
                        dk[db] = mma(aqt, df, dk[db]);
                    }
                }
            }
        }
    }

    if (!key_ok) return;
    const float scale = 1.f / sqrtf((float)D);
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
            f32x4 a, bq;
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = dk[db][4 * e4 + i] * scale; bq[i] = dv[db][4 * e4 + i]; }
            const int col = db * 32 + 8 * e4 + 4 * hh;
            *reinterpret_cast<f32x4 *>(dk_part + kv_off + col) = a;
            *reinterpret_cast<f32x4 *>(dv_part + kv_off + col) = bq;
        }
}

template <typename T, int D>
static hipError_t launch_bwd_d(const SegShape &s, const DropArgs &dr, const T *q, const T *k, const T *v, const T *out,
                               const float *lse, const T *dO, T *dq, float *dk_part, float *dv_part,
                               const Workspace &ws, hipStream_t st)
{
    hipError_t e;
    int n_splits = choose_splits(s.l_s, s.l_x, s.B, s.H, dq_rows_per_wg((int)sizeof(T), D));
    auto rowdot = [&]() -> hipError_t {
        const int64_t threads = (int64_t)s.B * s.l_s * s.H * 16;
        TimedLaunch tl(K_ROWDOT, st);
        hipLaunchKernelGGL((bwd_rowdot_kernel<T, D>), dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st,
                           s, out, dO, ws.D);
        return hipGetLastError();
    };
    auto generic_dq = [&](auto drop) -> hipError_t {
        using C = DqCfg<T, D>;
        dim3 grid((s.l_s + C::BR - 1) / C::BR, s.B * s.H, n_splits);
        TimedLaunch tl(K_DQ, st);
        hipLaunchKernelGGL((bwd_dq_kernel<T, D, decltype(drop)::value>), grid, dim3(C::NT), 0, st, s, dr, q, k, v, dO, lse,
                           ws.D, dq, ws.dq_part, n_splits);
        return hipGetLastError();
    };
    auto generic_dkv = [&](auto drop) -> hipError_t {
        using C = DkvCfg<T, D>;
        dim3 grid((s.l_x + C::BKV - 1) / C::BKV, s.B * s.H);
        TimedLaunch tl(K_DKV, st);
        hipLaunchKernelGGL((bwd_dkv_kernel<T, D, decltype(drop)::value>), grid, dim3(C::NT), 0, st, s, dr, q, k, v, dO, lse,
                           ws.D, dk_part, dv_part);
        return hipGetLastError();
    };
    if constexpr (sizeof(T) == 2) {
        // The dQ workgroups share their launch with the dK/dV ones and need not fill the chip alone:
        // keys are split only so far that a dQ workgroup (64 key tiles at most) does not outlast the
        // rest of the launch.  Never more splits than the workspace was sized for.  (Dropout runs
        // the same launch with the kernels' dropout variants.)
        const int64_t kv_extent = s.causal ? (s.s0 + s.l_s < s.l_x ? s.s0 + s.l_s : (int64_t)s.l_x) : (int64_t)s.l_x;
        const int want = (int)((kv_extent + 64 * 64 - 1) / (64 * 64));
        if (want < n_splits) n_splits = want < 1 ? 1 : want;
        if ((e = launch_bwd_bf16_main(s, dr, q, k, v, out, lse, dO, dq, dk_part, dv_part, ws, n_splits, st)) != hipSuccess)
            return e;
    } else {
        if ((e = rowdot()) != hipSuccess) return e;
        if (dr.thr != 0) {
            if ((e = generic_dq(std::true_type{})) != hipSuccess) return e;
            if ((e = generic_dkv(std::true_type{})) != hipSuccess) return e;
        } else {
            if ((e = generic_dq(std::false_type{})) != hipSuccess) return e;
            if ((e = generic_dkv(std::false_type{})) != hipSuccess) return e;
        }
    }
    if (n_splits > 1) {
        const int64_t n4 = (int64_t)s.B * s.l_s * s.H * D / 4;
        TimedLaunch tl(K_DQ_MERGE, st);
        hipLaunchKernelGGL((bwd_dq_merge_kernel<T>), dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st,
                           ws.dq_part, n_splits, n4, dq);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    return hipSuccess;
}

template <typename T>
hipError_t launch_bwd(const SegShape &s, const DropArgs &dr, const T *q, const T *k, const T *v, const T *out,
                      const float *lse, const T *dO, T *dq, float *dk_part, float *dv_part, const Workspace &ws,
                      hipStream_t st)
{
    if (s.d == 64) return launch_bwd_d<T, 64>(s, dr, q, k, v, out, lse, dO, dq, dk_part, dv_part, ws, st);
    return launch_bwd_d<T, 128>(s, dr, q, k, v, out, lse, dO, dq, dk_part, dv_part, ws, st);
}

template hipError_t launch_bwd<bf16_t>(const SegShape &, const DropArgs &, const bf16_t *, const bf16_t *, const bf16_t *,
                                       const bf16_t *, const float *, const bf16_t *, bf16_t *, float *, float *,
                                       const Workspace &, hipStream_t);
template hipError_t launch_bwd<float>(const SegShape &, const DropArgs &, const float *, const float *, const float *,
                                      const float *, const float *, const float *, float *, float *, float *,
                                      const Workspace &, hipStream_t);

} // namespace lss
