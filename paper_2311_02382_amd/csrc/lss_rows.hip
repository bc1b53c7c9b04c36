// Segment-local operations of a layer other than the self-attention (Section 3, Principles 1 and
// 2): each works on the rows of one sequence segment with no dependence on other segments.
//   positional embedding: a segment adds only its own contiguous rows of the lookup table
//   layer normalisation over the E_m columns of a row, with learned scale and shift
//   GeLU (exact, u Phi(u)) between the two linear transforms of the feed-forward unit
// All of it is streaming work bound by HBM bandwidth: bf16 activations, fp32 arithmetic, 16-byte
// accesses, one wavefront per row where a row needs a reduction.  Sums over rows (the gradients of
// the table rows, of gamma and of beta) are taken in a fixed order: no atomics.
#include "lss_common.h"
#include "lss_kernels.h"

#include <mutex>

namespace lss {

namespace {

__device__ __forceinline__ void unpack8(const bf16x8 &v, float (&f)[8])
{
#pragma unroll
    for (int e = 0; e < 8; ++e) f[e] = (float)v[e];
}
__device__ __forceinline__ bf16x8 pack8(const float (&f)[8])
{
    bf16x8 v;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (bf16_t)f[e];
    return v;
}
__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int sh = 32; sh >= 1; sh >>= 1) x += __shfl_xor(x, sh);
    return x;
}

// x[b, r, :] = tok[b, r, :] + pe[s0 + r, :]; one 16-byte chunk per thread
__global__ __launch_bounds__(256) void embed_pe_fwd_kernel(const bf16_t *__restrict__ tok, const bf16_t *__restrict__ pe,
                                                           int64_t s0, int l_s, int64_t n_chunks, int cpr,
                                                           bf16_t *__restrict__ x)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_chunks) return;
    const int64_t row = i / cpr;                // b * l_s + r
    const int c = (int)(i % cpr), r = (int)(row % l_s);
    float a[8], p[8];
    unpack8(*reinterpret_cast<const bf16x8 *>(tok + i * 8), a);
    unpack8(*reinterpret_cast<const bf16x8 *>(pe + ((s0 + r) * cpr + c) * 8), p);
#pragma unroll
    for (int e = 0; e < 8; ++e) a[e] += p[e];
    *reinterpret_cast<bf16x8 *>(x + i * 8) = pack8(a);
}

// dpe[r, :] = sum_b dx[b, r, :], b in increasing order; one 8-column chunk of a row per thread
__global__ __launch_bounds__(256) void embed_pe_bwd_kernel(const bf16_t *__restrict__ dx, int B, int l_s, int cpr,
                                                           float *__restrict__ dpe)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;       // r * cpr + c
    if (i >= (int64_t)l_s * cpr) return;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int b = 0; b < B; ++b) {
        float a[8];
        unpack8(*reinterpret_cast<const bf16x8 *>(dx + ((int64_t)b * l_s * cpr + i) * 8), a);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += a[e];
    }
    *reinterpret_cast<f32x4 *>(dpe + i * 8) = f32x4{acc[0], acc[1], acc[2], acc[3]};
    *reinterpret_cast<f32x4 *>(dpe + i * 8 + 4) = f32x4{acc[4], acc[5], acc[6], acc[7]};
}

// out = x + dropout(delta) (x may be null: the dropout alone); element (b, r, c) is decided like the
// attention weight of (batch*head b, global row s0 + r, key c).  One 16-byte chunk per thread.
template <bool DROP>
__global__ __launch_bounds__(256) void residual_add_kernel(const bf16_t *x, const bf16_t *delta, DropArgs dr, int64_t s0,
                                                           int l_s, int64_t n_chunks, int cpr, bf16_t *out)    // out may alias x or delta
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_chunks) return;
    float a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, dl[8];
    if (x) unpack8(*reinterpret_cast<const bf16x8 *>(x + i * 8), a);
    unpack8(*reinterpret_cast<const bf16x8 *>(delta + i * 8), dl);
    if constexpr (DROP) {
        const int64_t row = i / cpr;
        const uint32_t c0 = (uint32_t)(i % cpr) * 8u;
        const uint32_t rk = drop_row_key(dr.seed_lo, (uint32_t)(row / l_s), (uint32_t)(s0 + row % l_s));
        const uint32_t cs = drop_col_seed(dr.seed_hi);
#pragma unroll
        for (int e = 0; e < 8; ++e) dl[e] = drop_keep(rk, drop_col_key(cs, c0 + e), dr.thr) ? dl[e] * dr.scale : 0.f;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) a[e] += dl[e];
    *reinterpret_cast<bf16x8 *>(out + i * 8) = pack8(a);
}

constexpr int LN_MAXC = 8;      // 16-byte chunks a lane may hold: rows of up to 64 * 8 * 8 = 4096 columns

// One wavefront per row: the row is read once into registers (lane l holds chunks l, l + 64, ...
// of it, at most NCH of them: the kernels are compiled for NCH = 1, 2, 4, 8 and the narrowest that
// covers E runs), mean and variance are taken in two passes over the registers.
template <int NCH>
__global__ __launch_bounds__(256) void layernorm_fwd_kernel(const bf16_t *__restrict__ x, const float *__restrict__ gamma,
                                                            const float *__restrict__ beta, float eps, int64_t rows, int E,
                                                            bf16_t *__restrict__ y, float *__restrict__ mean,
                                                            float *__restrict__ rstd)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int cpr = E / 8;
    float v[NCH][8];
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
        const int c = lane + 64 * k;
        if (c < cpr) {
            unpack8(*reinterpret_cast<const bf16x8 *>(x + (row * cpr + c) * 8), v[k]);
#pragma unroll
            for (int e = 0; e < 8; ++e) s += v[k][e];
        }
    }
    const float mu = wave_sum(s) / (float)E;
    float q = 0.f;
#pragma unroll
    for (int k = 0; k < NCH; ++k)
        if (lane + 64 * k < cpr) {
#pragma unroll
            for (int e = 0; e < 8; ++e) { const float dlt = v[k][e] - mu; q += dlt * dlt; }
        }
    const float rs = 1.0f / sqrtf(wave_sum(q) / (float)E + eps);
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
        const int c = lane + 64 * k;
        if (c < cpr) {
            float o[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (v[k][e] - mu) * rs * gamma[c * 8 + e] + beta[c * 8 + e];
            *reinterpret_cast<bf16x8 *>(y + (row * cpr + c) * 8) = pack8(o);
        }
    }
    if (lane == 0) { mean[row] = mu; rstd[row] = rs; }
}

// Backward of the above.  A workgroup owns LN_ROWS consecutive rows, one wavefront walks every
// fourth of them: dx of a row needs two row sums; the contributions to dgamma and dbeta stay in the
// lane that owns the columns and are added up over the wavefront's rows in row order, then over the
// four wavefronts in wavefront order (through LDS) into part[workgroup] -- a second kernel adds
// the workgroups' parts in a fixed order.
constexpr int LN_ROWS = 32;
template <int NCH>
__global__ __launch_bounds__(256) void layernorm_bwd_kernel(const bf16_t *__restrict__ x, const float *__restrict__ gamma,
                                                            const float *__restrict__ mean, const float *__restrict__ rstd,
                                                            const bf16_t *__restrict__ dy, int64_t rows, int E,
                                                            bf16_t *__restrict__ dx, float *__restrict__ part)
{
    extern __shared__ float red[];              // [4][2][E]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cpr = E / 8;
    float dg[NCH][8], db[NCH][8];
#pragma unroll
    for (int k = 0; k < NCH; ++k)
#pragma unroll
        for (int e = 0; e < 8; ++e) { dg[k][e] = 0.f; db[k][e] = 0.f; }
    const int64_t row0 = (int64_t)blockIdx.x * LN_ROWS;
    for (int i = wave; i < LN_ROWS; i += 4) {
        const int64_t row = row0 + i;
        if (row >= rows) break;
        const float mu = mean[row], rs = rstd[row];
        float xh[NCH][8], g[NCH][8];
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int k = 0; k < NCH; ++k) {
            const int c = lane + 64 * k;
            if (c < cpr) {
                float xv[8], dv[8];
                unpack8(*reinterpret_cast<const bf16x8 *>(x + (row * cpr + c) * 8), xv);
                unpack8(*reinterpret_cast<const bf16x8 *>(dy + (row * cpr + c) * 8), dv);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    xh[k][e] = (xv[e] - mu) * rs;
                    g[k][e] = dv[e] * gamma[c * 8 + e];
                    s1 += g[k][e];
                    s2 += g[k][e] * xh[k][e];
                    dg[k][e] += dv[e] * xh[k][e];
                    db[k][e] += dv[e];
                }
            }
        }
        const float m1 = wave_sum(s1) / (float)E, m2 = wave_sum(s2) / (float)E;
#pragma unroll
        for (int k = 0; k < NCH; ++k) {
            const int c = lane + 64 * k;
            if (c < cpr) {
                float o[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = rs * (g[k][e] - m1 - xh[k][e] * m2);
                *reinterpret_cast<bf16x8 *>(dx + (row * cpr + c) * 8) = pack8(o);
            }
        }
    }
#pragma unroll
    for (int k = 0; k < NCH; ++k) {
        const int c = lane + 64 * k;
        if (c < cpr) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                red[(wave * 2 + 0) * E + c * 8 + e] = dg[k][e];
                red[(wave * 2 + 1) * E + c * 8 + e] = db[k][e];
            }
        }
    }
    __syncthreads();
    for (int col = threadIdx.x; col < 2 * E; col += 256) {
        const int which = col / E, cc = col % E;
        float acc = red[(0 * 2 + which) * E + cc];
#pragma unroll
        for (int w = 1; w < 4; ++w) acc += red[(w * 2 + which) * E + cc];
        part[((int64_t)blockIdx.x * 2 + which) * E + cc] = acc;
    }
}
// 64 columns x 16 groups of parts per workgroup: thread (group pg, chunk cc) adds parts pg, pg + 16, ...
// of its four columns in increasing order, then the 16 group sums are added in group order.
__global__ __launch_bounds__(256) void layernorm_bwd_params_kernel(const float *__restrict__ part, int n_parts, int E,
                                                                   float *__restrict__ dgamma, float *__restrict__ dbeta)
{
    __shared__ f32x4 red[16][16];
    const int cc = threadIdx.x & 15, pg = threadIdx.x >> 4;
    const int col = (blockIdx.x * 16 + cc) * 4;         // [0, 2E): dgamma's columns, then dbeta's
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    if (col < 2 * E)
        for (int p = pg; p < n_parts; p += 16) acc += *reinterpret_cast<const f32x4 *>(part + (int64_t)p * 2 * E + col);
    red[pg][cc] = acc;
    __syncthreads();
    if (pg == 0 && col < 2 * E) {
#pragma unroll
        for (int j = 1; j < 16; ++j) acc += red[j][cc];
        *reinterpret_cast<f32x4 *>(col < E ? dgamma + col : dbeta + (col - E)) = acc;
    }
}

// g = GeLU(u) = u Phi(u);  du = dg * (Phi(u) + u phi(u)).  One 16-byte chunk per thread.
__global__ __launch_bounds__(256) void gelu_fwd_kernel(const bf16_t *__restrict__ u, int64_t n_chunks, bf16_t *__restrict__ g)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_chunks) return;
    float a[8];
    unpack8(*reinterpret_cast<const bf16x8 *>(u + i * 8), a);
#pragma unroll
    for (int e = 0; e < 8; ++e) a[e] = gelu_value(a[e]);
    *reinterpret_cast<bf16x8 *>(g + i * 8) = pack8(a);
}
__global__ __launch_bounds__(256) void gelu_bwd_kernel(const bf16_t *__restrict__ u, const bf16_t *__restrict__ dg,
                                                       int64_t n_chunks, bf16_t *__restrict__ du)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_chunks) return;
    float a[8], d[8];
    unpack8(*reinterpret_cast<const bf16x8 *>(u + i * 8), a);
    unpack8(*reinterpret_cast<const bf16x8 *>(dg + i * 8), d);
#pragma unroll
    for (int e = 0; e < 8; ++e) d[e] *= gelu_slope(a[e]);
    *reinterpret_cast<bf16x8 *>(du + i * 8) = pack8(d);
}

unsigned blocks_for(int64_t n) { return (unsigned)((n + 255) / 256); }

} // namespace

hipError_t launch_embed_pe_fwd(const bf16_t *tok, const bf16_t *pe, int64_t s0, int l_s, int B, int E, bf16_t *x,
                               hipStream_t st)
{
    const int64_t n = (int64_t)B * l_s * (E / 8);
    if (n == 0) return hipSuccess;
    TimedLaunch tl(K_PE_FWD, st);
    hipLaunchKernelGGL(embed_pe_fwd_kernel, dim3(blocks_for(n)), dim3(256), 0, st, tok, pe, s0, l_s, n, E / 8, x);
    return hipGetLastError();
}
hipError_t launch_embed_pe_bwd(const bf16_t *dx, int l_s, int B, int E, float *dpe, hipStream_t st)
{
    const int64_t n = (int64_t)l_s * (E / 8);
    if (n == 0) return hipSuccess;
    TimedLaunch tl(K_PE_BWD, st);
    hipLaunchKernelGGL(embed_pe_bwd_kernel, dim3(blocks_for(n)), dim3(256), 0, st, dx, B, l_s, E / 8, dpe);
    return hipGetLastError();
}
hipError_t launch_residual_add(const bf16_t *x, const bf16_t *delta, const DropArgs &drop, int64_t s0, int l_s, int B, int E,
                               bf16_t *out, hipStream_t st)
{
    const int64_t n = (int64_t)B * l_s * (E / 8);
    if (n == 0) return hipSuccess;
    TimedLaunch tl(K_RESIDUAL, st);
    if (drop.thr != 0)
        hipLaunchKernelGGL(residual_add_kernel<true>, dim3(blocks_for(n)), dim3(256), 0, st, x, delta, drop, s0, l_s, n, E / 8, out);
    else
        hipLaunchKernelGGL(residual_add_kernel<false>, dim3(blocks_for(n)), dim3(256), 0, st, x, delta, drop, s0, l_s, n, E / 8, out);
    return hipGetLastError();
}
int layernorm_max_columns() { return 64 * LN_MAXC * 8; }
size_t layernorm_bwd_scratch_bytes(int64_t rows, int E) { return (size_t)((rows + LN_ROWS - 1) / LN_ROWS) * 2 * E * sizeof(float); }
hipError_t launch_layernorm_fwd(const bf16_t *x, const float *gamma, const float *beta, float eps, int64_t rows, int E,
                                bf16_t *y, float *mean, float *rstd, hipStream_t st)
{
    if (rows == 0) return hipSuccess;
    TimedLaunch tl(K_LN_FWD, st);
    const dim3 grid((unsigned)((rows + 3) / 4));
#define LSS_LN_FWD(NCH) hipLaunchKernelGGL(layernorm_fwd_kernel<NCH>, grid, dim3(256), 0, st, x, gamma, beta, eps, rows, E, y, mean, rstd)
    if (E <= 512) LSS_LN_FWD(1);
    else if (E <= 1024) LSS_LN_FWD(2);
    else if (E <= 2048) LSS_LN_FWD(4);
    else LSS_LN_FWD(8);
#undef LSS_LN_FWD
    return hipGetLastError();
}
hipError_t launch_layernorm_bwd(const bf16_t *x, const float *gamma, const float *mean, const float *rstd, const bf16_t *dy,
                                int64_t rows, int E, bf16_t *dx, float *dgamma, float *dbeta, float *scratch, hipStream_t st)
{
    const int n_parts = (int)((rows + LN_ROWS - 1) / LN_ROWS);
    if (rows > 0) {
        // the widest variant's LDS (4 wavefronts x 2 x E floats) exceeds the default limit
        static std::once_flag once;
        static hipError_t attr = hipSuccess;
        std::call_once(once, [] {
            attr = hipFuncSetAttribute(reinterpret_cast<const void *>(layernorm_bwd_kernel<8>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 8 * 64 * LN_MAXC * 8 * (int)sizeof(float));
        });
        if (attr != hipSuccess) return attr;
        TimedLaunch tl(K_LN_BWD, st);
        const dim3 grid((unsigned)n_parts);
        const size_t lds = (size_t)8 * E * sizeof(float);
#define LSS_LN_BWD(NCH) hipLaunchKernelGGL(layernorm_bwd_kernel<NCH>, grid, dim3(256), lds, st, x, gamma, mean, rstd, dy, rows, E, dx, scratch)
        if (E <= 512) LSS_LN_BWD(1);
        else if (E <= 1024) LSS_LN_BWD(2);
        else if (E <= 2048) LSS_LN_BWD(4);
        else LSS_LN_BWD(8);
#undef LSS_LN_BWD
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    TimedLaunch tl(K_LN_PARAMS, st);
    hipLaunchKernelGGL(layernorm_bwd_params_kernel, dim3((unsigned)((2 * E + 63) / 64)), dim3(256), 0, st, scratch, n_parts, E,
                       dgamma, dbeta);
    return hipGetLastError();
}
hipError_t launch_gelu_fwd(const bf16_t *u, int64_t n, bf16_t *g, hipStream_t st)
{
    if (n == 0) return hipSuccess;
    TimedLaunch tl(K_GELU_FWD, st);
    hipLaunchKernelGGL(gelu_fwd_kernel, dim3(blocks_for(n / 8)), dim3(256), 0, st, u, n / 8, g);
    return hipGetLastError();
}
hipError_t launch_gelu_bwd(const bf16_t *u, const bf16_t *dg, int64_t n, bf16_t *du, hipStream_t st)
{
    if (n == 0) return hipSuccess;
    TimedLaunch tl(K_GELU_BWD, st);
    hipLaunchKernelGGL(gelu_bwd_kernel, dim3(blocks_for(n / 8)), dim3(256), 0, st, u, dg, n / 8, du);
    return hipGetLastError();
}

} // namespace lss
