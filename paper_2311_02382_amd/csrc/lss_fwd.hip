// Forward of Eq. 2 (Section 3, Principle 3) for one segment: E_i = softmax(Q_i K^T / sqrt(d)) V.
//
// A workgroup of 4 wavefronts owns 128 query rows (32 per wavefront) of one (batch, head)
// and walks over key tiles of 64 rows; grid.z splits a tile range among workgroups.
// Per key tile:   S^T = K Q^T   (A = K rows from LDS, B = the wavefront's Q rows in registers)
// so one lane holds ONE query column and 16 keys per 32-key block: every per-query
// quantity of the online softmax (running max, running sum, rescale factor) is a per-lane
// scalar, and the only cross-lane step is between the two halves of the wavefront.
// Then            O^T += V^T P^T (A = V^T from a transposed LDS tile, B = P^T straight from
// the S^T registers, see lss_common.h).
#include "lss_common.h"
#include "lss_kernels.h"

namespace lss {

template <typename T, int D>
struct FwdCfg {
    static constexpr int BR = 128, BC = 64, NT = 256;
    static constexpr int E = Elems16<T>::n;
    static constexpr int KP = D + E;    // pitch of the row-major K tile
    static constexpr int VP = BC + E;   // pitch of the transposed V tile
};

template <typename T, int D, bool DROP>
__global__ __launch_bounds__(256) void fwd_kernel(SegShape s, DropArgs dr, const T *__restrict__ q,
                                                  const T *__restrict__ k, const T *__restrict__ v,
                                                  T *__restrict__ out, float *__restrict__ lse,
                                                  float *__restrict__ o_part,
                                                  float *__restrict__ lse_part, int n_splits)
{
    using C = FwdCfg<T, D>;
    __shared__ __attribute__((aligned(16))) T sK[C::BC * C::KP];
    __shared__ __attribute__((aligned(16))) T sVt[D * C::VP];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lq = lane & 31, hh = lane >> 5;
    const int bh = blockIdx.y, b = bh / s.H, h = bh % s.H, split = blockIdx.z;
    const int r0 = blockIdx.x * C::BR;
    const int r = r0 + wave * 32 + lq;          // this lane's query row (local)
    const bool row_ok = r < s.l_s;
    const int64_t g = s.s0 + r;                 // its global position
    const int64_t ld = (int64_t)s.H * D;        // row stride of every activation

    // keys any row of this tile can see, and this workgroup's share of their tiles
    const int r_last = min(r0 + C::BR, s.l_s) - 1;
    const int kv_end = s.causal ? (int)min<int64_t>(s.l_x, s.s0 + r_last + 1) : s.l_x;
    const int n_tiles = (kv_end + C::BC - 1) / C::BC;
    const int per = (n_tiles + n_splits - 1) / n_splits;
    const int t_begin = split * per, t_end = min(n_tiles, t_begin + per);

    Frag<T> qf[D / 16];
    {
        const T *qp = q + ((int64_t)b * s.l_s + r) * ld + (int64_t)h * D + hh * 8;
#pragma unroll
        for (int kb = 0; kb < D / 16; ++kb) qf[kb] = row_ok ? load_frag<T>(qp + kb * 16) : zero_frag<T>();
    }

    f32x16 o[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[db][e] = 0.f;
    float m = -INFINITY, l = 0.f;               // running max (log2 domain) and sum, per query
    const float c = kLog2e / sqrtf((float)D);   // score -> log2 domain
    uint32_t drop_rk = 0u, drop_cs = 0u;        // dropout: the key of this lane's global row; the column seed
    if (DROP) { drop_rk = drop_row_key(dr.seed_lo, (uint32_t)bh, (uint32_t)g); drop_cs = drop_col_seed(dr.seed_hi); }

    const T *kbase = k + (int64_t)b * s.l_x * ld + (int64_t)h * D;
    const T *vbase = v + (int64_t)b * s.l_x * ld + (int64_t)h * D;

    for (int t = t_begin; t < t_end; ++t) {
        const int j0 = t * C::BC;
        __syncthreads();
        load_tile<T, D, C::BC, C::NT, C::KP, 0, true, false>(kbase + (int64_t)j0 * ld, ld, s.l_x - j0, sK, nullptr, tid);
        load_tile<T, D, C::BC, C::NT, 0, C::VP, false, true>(vbase + (int64_t)j0 * ld, ld, s.l_x - j0, nullptr, sVt, tid);
        __syncthreads();

        f32x16 sc[2];
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2) {
#pragma unroll
            for (int e = 0; e < 16; ++e) sc[kb2][e] = 0.f;
#pragma unroll
            for (int kb = 0; kb < D / 16; ++kb) {
                const Frag<T> a = load_frag<T>(&sK[(kb2 * 32 + lq) * C::KP + kb * 16 + hh * 8]);
                sc[kb2] = mma(a, qf[kb], sc[kb2]);
            }
        }

        // mask: keys past the end of the sequence, and (causal) keys after the query.
        const bool tail = j0 + C::BC > s.l_x;
        const bool diag = s.causal && (j0 + C::BC - 1 > s.s0 + r0 + wave * 32);
        if (tail || diag) {
#pragma unroll
            for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int key = j0 + kb2 * 32 + 8 * (e >> 2) + 4 * hh + (e & 3);
                    if (key >= s.l_x || (s.causal && key > g)) sc[kb2][e] = -INFINITY;
                }
        }

        float mx = -INFINITY;
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
            for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sc[kb2][e]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m, mx * c);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = fast_exp2(m - m_use);
        float psum = 0.f;
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float p = fast_exp2(sc[kb2][e] * c - m_use);
                psum += p;          // the row sum (hence lse and the normalisation) is that of the softmax
                if (DROP) {         // the weight that multiplies V is dropped or scaled by 1 / (1 - p_drop)
                    const int key = j0 + kb2 * 32 + 8 * (e >> 2) + 4 * hh + (e & 3);
                    sc[kb2][e] = drop_keep(drop_rk, drop_col_key(drop_cs, (uint32_t)key), dr.thr) ? p * dr.scale : 0.f;
                } else {
                    sc[kb2][e] = p;
                }
            }
        l = l * alpha + psum;       // each half keeps the sum of its own keys
        m = m_new;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[db][e] *= alpha;

#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const Frag<T> pf = acc_to_frag<T>(sc[ks >> 1], ks & 1);
#pragma unroll
            for (int db = 0; db < D / 32; ++db) {
                const Frag<T> a = load_frag<T>(&sVt[(db * 32 + lq) * C::VP + ks * 16 + hh * 8]);
                o[db] = mma(a, pf, o[db]);
            }
        }
    }

    const float l_tot = l + __shfl_xor(l, 32);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    const float lse_nat = l_tot > 0.f ? (m + log2f(l_tot)) * kLn2 : -INFINITY;
    if (!row_ok) return;

    if (n_splits == 1) {
        T *op = out + ((int64_t)b * s.l_s + r) * ld + (int64_t)h * D;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                T *dst = op + db * 32 + 8 * e4 + 4 * hh;
#pragma unroll
                for (int i = 0; i < 4; ++i) dst[i] = (T)(o[db][4 * e4 + i] * inv);
            }
        if (hh == 0) lse[(int64_t)bh * s.l_s + r] = lse_nat;
    } else {
        const int64_t row = ((int64_t)split * gridDim.y + bh) * s.l_s + r;
        float *op = o_part + row * D;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                f32x4 val;
#pragma unroll
                for (int i = 0; i < 4; ++i) val[i] = o[db][4 * e4 + i] * inv;
                *reinterpret_cast<f32x4 *>(op + db * 32 + 8 * e4 + 4 * hh) = val;
            }
        if (hh == 0) lse_part[row] = lse_nat;
    }
}

// Fixed-order merge of the split-KV partial results of one query row:
//   lse = log sum_s exp(lse_s),  out = sum_s exp(lse_s - lse) out_s.
// One thread per (b*H + h, r, group of 4 columns).
// MAXS: compile-time bound of n_splits (loop unrolling; all loads of a thread issued together)
template <typename T, int D, int MAXS>
__global__ __launch_bounds__(256) void fwd_merge_kernel(SegShape s, const float *__restrict__ o_part,
                                                        const float *__restrict__ lse_part, int n_splits,
                                                        T *__restrict__ out, float *__restrict__ lse)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t rows = (int64_t)s.B * s.H * s.l_s;
    if (idx >= rows * (D / 4)) return;
    const int64_t row = idx / (D / 4);
    const int c4 = (int)(idx % (D / 4)) * 4;
    // all loads of a thread are independent: issue them together, then combine in split order
    float l[MAXS];
    f32x4 part[MAXS];
#pragma unroll
    for (int sp = 0; sp < MAXS; ++sp) {
        const int spc = sp < n_splits ? sp : n_splits - 1;
        l[sp] = __builtin_nontemporal_load(lse_part + spc * rows + row);
        if constexpr (sizeof(T) == 2) {     // the bf16 kernel writes its partial outputs in bf16
            const bf16x4 pv = __builtin_nontemporal_load(
                reinterpret_cast<const bf16x4 *>(reinterpret_cast<const bf16_t *>(o_part) + (spc * rows + row) * D + c4));
#pragma unroll
            for (int i = 0; i < 4; ++i) part[sp][i] = (float)pv[i];
        } else {
            part[sp] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(o_part + (spc * rows + row) * D + c4));
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int sp = 0; sp < MAXS; ++sp)
        if (sp < n_splits) mx = fmaxf(mx, l[sp]);
    float sum = 0.f;
#pragma unroll
    for (int sp = 0; sp < MAXS; ++sp)
        if (sp < n_splits) sum += expf(l[sp] - mx);
    const float total = mx + logf(sum);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int sp = 0; sp < MAXS; ++sp)
        if (sp < n_splits) acc += expf(l[sp] - total) * part[sp];
    const int r = (int)(row % s.l_s);
    const int64_t bh = row / s.l_s;
    const int64_t b = bh / s.H, h = bh % s.H;
    T *dst = out + ((b * s.l_s + r) * s.H + h) * D + c4;
#pragma unroll
    for (int i = 0; i < 4; ++i) dst[i] = (T)acc[i];
    if (c4 == 0) lse[row] = total;
}

template <typename T, int D>
static hipError_t launch_fwd_d(const SegShape &s, const DropArgs &drop, const T *q, const T *k, const T *v, T *out,
                               float *lse, const Workspace &ws, hipStream_t st)
{
    using C = FwdCfg<T, D>;
    // Under the causal mask a segment near the start of the sequence sees few keys: the split count
    // follows the keys this segment's query tiles see, within what the workspace was sized for.
    const int rows_per_wg = fwd_rows_per_wg((int)sizeof(T), D);
    const int64_t kv_extent = s.causal ? (s.s0 + s.l_s < s.l_x ? s.s0 + s.l_s : (int64_t)s.l_x) : (int64_t)s.l_x;
    const int n_splits = pick_fwd_splits(s.l_s, s.B, s.H, rows_per_wg, (kv_extent + 63) / 64,
                                         max_fwd_splits(s.l_s, s.l_x, s.B, s.H, rows_per_wg), fwd_wgs_per_cu((int)sizeof(T), D));
    hipError_t e;
    const dim3 grid((s.l_s + C::BR - 1) / C::BR, s.B * s.H, n_splits);
    if constexpr (sizeof(T) == 2) {
        e = launch_fwd_bf16_main(s, drop, q, k, v, out, lse, ws, n_splits, st);
    } else if (drop.thr != 0) {
        TimedLaunch tl(K_FWD, st);
        hipLaunchKernelGGL((fwd_kernel<T, D, true>), grid, dim3(C::NT), 0, st, s, drop, q, k, v, out, lse, ws.o_part,
                           ws.lse_part, n_splits);
        e = hipGetLastError();
    } else {
        TimedLaunch tl(K_FWD, st);
        hipLaunchKernelGGL((fwd_kernel<T, D, false>), grid, dim3(C::NT), 0, st, s, drop, q, k, v, out, lse, ws.o_part,
                           ws.lse_part, n_splits);
        e = hipGetLastError();
    }
    if (e != hipSuccess || n_splits == 1) return e;
    const int64_t items = (int64_t)s.B * s.H * s.l_s * (D / 4);
    {
        TimedLaunch tl(K_FWD_MERGE, st);
        const dim3 grid((unsigned)((items + 255) / 256)), block(256);
        if (n_splits <= 2)
            hipLaunchKernelGGL((fwd_merge_kernel<T, D, 2>), grid, block, 0, st, s, ws.o_part, ws.lse_part, n_splits, out, lse);
        else if (n_splits <= 4)
            hipLaunchKernelGGL((fwd_merge_kernel<T, D, 4>), grid, block, 0, st, s, ws.o_part, ws.lse_part, n_splits, out, lse);
        else if (n_splits <= 8)
            hipLaunchKernelGGL((fwd_merge_kernel<T, D, 8>), grid, block, 0, st, s, ws.o_part, ws.lse_part, n_splits, out, lse);
        else
            hipLaunchKernelGGL((fwd_merge_kernel<T, D, 16>), grid, block, 0, st, s, ws.o_part, ws.lse_part, n_splits, out, lse);
    }
    return hipGetLastError();
}

template <typename T>
hipError_t launch_fwd(const SegShape &s, const DropArgs &drop, const T *q, const T *k, const T *v, T *out, float *lse,
                      const Workspace &ws, hipStream_t st)
{
    if (s.d == 64) return launch_fwd_d<T, 64>(s, drop, q, k, v, out, lse, ws, st);
    return launch_fwd_d<T, 128>(s, drop, q, k, v, out, lse, ws, st);
}

template hipError_t launch_fwd<bf16_t>(const SegShape &, const DropArgs &, const bf16_t *, const bf16_t *, const bf16_t *,
                                       bf16_t *, float *, const Workspace &, hipStream_t);
template hipError_t launch_fwd<float>(const SegShape &, const DropArgs &, const float *, const float *, const float *, float *,
                                      float *, const Workspace &, hipStream_t);

} // namespace lss
