// Segment sum of the per-segment dK/dV partials -- the arithmetic of the reduce-scatter
// that is the backward of the all-gather (Section 3, Principle 4, Fig. 2(v)):
//     out = parts[0] + parts[1] + ... + parts[n-1], elementwise, in that order.
// Pure streaming work, bound by HBM bandwidth: each thread owns 4 consecutive floats and
// adds the parts in index order, skipping (without reading) rows a part declares empty.
#include "lss_common.h"
#include "lss_kernels.h"

namespace lss {

struct ReduceArgs {
    const float *parts[kMaxReduceParts];
    int rows_valid[kMaxReduceParts];
    int n;
    int accumulate;     // 1: start from what `out` already holds (later chunks of a long list)
};

__global__ __launch_bounds__(256) void reduce_partials_kernel(ReduceArgs a, int64_t n4, int l_x, int row_f4,
                                                              float *__restrict__ out)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
        const int row = (int)((i / row_f4) % l_x);      // key row of this float4
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        if (a.accumulate) acc = *reinterpret_cast<const f32x4 *>(out + i * 4);
        // four parts at a time: the loads are independent and issued together, the adds keep list order
        int p = 0;
        for (; p + 4 <= a.n; p += 4) {
            f32x4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                v[u] = f32x4{0.f, 0.f, 0.f, 0.f};
                if (row < a.rows_valid[p + u]) v[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(a.parts[p + u] + i * 4));
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) acc += v[u];
        }
        for (; p < a.n; ++p)
            if (row < a.rows_valid[p]) acc += __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(a.parts[p] + i * 4));
        *reinterpret_cast<f32x4 *>(out + i * 4) = acc;
    }
}

hipError_t launch_reduce(const float *const *parts, int n, const int64_t *rows_valid, int64_t l_x, int64_t B,
                         int64_t H, int64_t d, float *out, hipStream_t st)
{
    const int64_t n4 = B * l_x * H * d / 4;
    if (n4 == 0) return hipSuccess;
    const int row_f4 = (int)(H * d / 4);
    const unsigned blocks = (unsigned)((n4 + 255) / 256 < 256 * 32 ? (n4 + 255) / 256 : 256 * 32);
    for (int first = 0; first < n; first += kMaxReduceParts) {
        ReduceArgs a;
        a.n = n - first < kMaxReduceParts ? n - first : kMaxReduceParts;
        a.accumulate = first > 0;
        for (int p = 0; p < a.n; ++p) {
            a.parts[p] = parts[first + p];
            const int64_t rv = rows_valid ? rows_valid[first + p] : l_x;
            a.rows_valid[p] = (int)(rv < 0 ? 0 : (rv > l_x ? l_x : rv));
        }
        TimedLaunch tl(K_REDUCE, st);
        hipLaunchKernelGGL(reduce_partials_kernel, dim3(blocks), dim3(256), 0, st, a, n4, (int)l_x, row_f4, out);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

} // namespace lss
