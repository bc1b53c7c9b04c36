// Issue-rate microbenchmarks for gfx950 (MI355X): the hardware facts the attention kernels' design leans on.
// A stand-alone program, not part of liblss_attn.so and not part of the paper's method:
//
//     python -m paper_2311_02382_amd.build --microbench && ./paper_2311_02382_amd/lss_microbench
//
// Sections
//   1. matrix pipe alone: cycles per V_MFMA_F32_32X32X16_BF16, the resulting ceiling in TFLOP/s and the clock
//      the chip sustains under that load (shader-clock counter against wall time);
//   2. vector issue: independent fma / exp2 streams from 1..4 wavefronts per SIMD;
//   3. co-issue: per matrix instruction NV fma + NT exp2 (+ NS scalar instructions), all independent:
//      how much vector (and scalar) work hides under a matrix instruction;
//   5. co-issue with LDS reads: per matrix instruction 3 fma + 1 exp2 and NL DS_READ_B128 whose data feeds the matrix
//      instructions of the NEXT iteration (two register sets, explicit waits), so only their issue and the LDS
//      pipeline count, not their latency;
//   6. the matrix pipe's sustained rate against the DATA and the instruction mix: the same loop of matrix instructions
//      on constant operands (all ones) and on random ones, then on random ones with the vector work of a softmax
//      beside each matrix instruction; every launch is long enough (10 ms) for the chip's power management to settle
//      the clock, and the figure is wall time, so it includes that clock;
//   4. LDS fragment reads: DS_READ_B128 by rows and DS_READ_B64_TR_B16 (transposing) on tiles with 128- and
//      256-byte rows under the chunk permutations of lss_bf16.h (tile_swizzle) and under the plain r & 7 one.
// Every kernel touches only registers and its own LDS; cycle counts come from clock64() of one wavefront.
#include <hip/hip_runtime.h>
#include <chrono>
#include <stdio.h>
#include <stdlib.h>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

#define CHECK(x)                                                                            \
    do {                                                                                    \
        hipError_t e_ = (x);                                                                \
        if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } \
    } while (0)

// ---- sections 1-3: per loop iteration 4 x (NM ? mfma : nothing, NV fma, NT exp2, 2*NS scalar ops), independent chains
template <int NM, int NV, int NT, int NS>
__global__ void issue_kernel(float *out, long long *cyc, int iters)
{
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(threadIdx.x * 0.001f); b[i] = (__bf16)1.0f; }
    f32x16 c[4];
    for (int j = 0; j < 4; ++j) for (int i = 0; i < 16; ++i) c[j][i] = 0.f;
    float x[16], y[16];
    for (int i = 0; i < 16; ++i) { x[i] = threadIdx.x * 1e-3f + i; y[i] = threadIdx.x * 1e-4f + i * 0.01f; }
    const float fa = 1.0001f, fb = 1e-4f;
    int sa = 1, sb = 2, sc = 3, sd = 4;
    __syncthreads();
    const long long t0 = clock64();
    for (int it = 0; it < iters; ++it) {
        int vi = 0, ti = 0;
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            if (NM) c[m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[m & 3], 0, 0, 0);
#pragma unroll
            for (int j = 0; j < NV; ++j) { x[vi & 15] = __builtin_fmaf(x[vi & 15], fa, fb); ++vi; }
#pragma unroll
            for (int j = 0; j < NT; ++j) { y[ti & 15] = __builtin_amdgcn_exp2f(y[ti & 15]); ++ti; }
#pragma unroll
            for (int j = 0; j < NS; ++j) {
                asm volatile("s_add_i32 %0, %0, %1" : "+s"(sa) : "s"(sb) : "scc");
                asm volatile("s_xor_b32 %0, %0, %1" : "+s"(sc) : "s"(sd) : "scc");
            }
        }
    }
    const long long t1 = clock64();
    float s = (float)(sa + sc);
    for (int i = 0; i < 16; ++i) s += x[i] + y[i];
    for (int j = 0; j < 4; ++j) s += c[j][j];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
    if ((threadIdx.x & 63) == 0 && blockIdx.x == 0) {
        atomicMin((unsigned long long *)&cyc[0], (unsigned long long)t0);
        atomicMax((unsigned long long *)&cyc[1], (unsigned long long)t1);
    }
}

template <int NM, int NV, int NT, int NS>
static void run_issue(float *d, long long *dc, const char *name)
{
    const int iters = 4000;
    printf("%-44s", name);
    for (int w = 1; w <= 4; ++w) {      // w wavefronts per SIMD: one workgroup of 256 w threads per compute unit
        issue_kernel<NM, NV, NT, NS><<<256, 256 * w>>>(d, dc, iters);
        CHECK(hipDeviceSynchronize());
        long long init[2] = {0x7fffffffffffffffLL, 0};
        CHECK(hipMemcpy(dc, init, 16, hipMemcpyHostToDevice));
        const auto w0 = std::chrono::steady_clock::now();
        issue_kernel<NM, NV, NT, NS><<<256, 256 * w>>>(d, dc, iters);
        CHECK(hipDeviceSynchronize());
        const double wall_us = std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - w0).count();
        long long cc[2];
        CHECK(hipMemcpy(cc, dc, 16, hipMemcpyDeviceToHost));
        const double per_slot = (double)(cc[1] - cc[0]) / iters / 4 / w;    // SIMD cycles per (mfma + its vector work) of one wavefront
        if (NM) printf("  w%d %5.1f (%3.0f%%)", w, per_slot, 100.0 * 32.0 / per_slot);
        else printf("  w%d %5.1f      ", w, per_slot);
        if (NM == 1 && NV == 0 && NT == 0 && NS == 0 && w == 4) {
            // ceiling: 256 CUs x 4 SIMDs x one 32x32x16 instruction (32768 flop) per `per_slot` cycles at the clock implied by wall time
            const double flops = 256.0 * 4 * w * iters * 4 * 32768.0;
            printf("\n    -> pure matrix loop: %.0f TFLOP/s over the launch's wall time (%.0f us incl. launch), ", flops / (wall_us * 1e-6) / 1e12, wall_us);
            printf("shader clock >= %.2f GHz", (double)(cc[1] - cc[0]) / (wall_us * 1e3));
        }
    }
    printf("\n");
}

// ---- section 5: matrix instructions fed from LDS one iteration ahead
template <int NL>
__global__ __launch_bounds__(512) void lds_issue_kernel(float *out, long long *cyc, int iters)
{
    __shared__ __attribute__((aligned(1024))) char smem[32 * 1024];
    for (int i = threadIdx.x; i < 32 * 1024 / 4; i += blockDim.x) reinterpret_cast<float *>(smem)[i] = (float)(i & 63) * 0.01f;
    const int lane = threadIdx.x & 63;
    bf16x8 b;
    for (int i = 0; i < 8; ++i) b[i] = (__bf16)1.0f;
    f32x16 c[4];
    for (int j = 0; j < 4; ++j) for (int i = 0; i < 16; ++i) c[j][i] = 0.f;
    float x[16], y[16];
    for (int i = 0; i < 16; ++i) { x[i] = threadIdx.x * 1e-3f + i; y[i] = threadIdx.x * 1e-4f + i * 0.01f; }
    const float fa = 1.0001f, fb = 1e-4f;
    const uint32_t addr = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char *)smem + (lane & 31) * 128 + (((lane >> 5) ^ lane) & 7) * 16;
    static_assert(NL <= 1, "one read per matrix instruction at most: more would need spills, and the compiler does not know\n"
                           "that a read issued from inline assembly is asynchronous");
    f32x4 f[2][4];      // two sets of 4 fragments (one per slot)
    for (int s2 = 0; s2 < 2; ++s2) for (int i = 0; i < 4; ++i) f[s2][i] = f32x4{0.f, 0.f, 0.f, 0.f};
    __syncthreads();
    const long long t0 = clock64();
    for (int it = 0; it < iters; it += 2) {
#pragma unroll
        for (int par = 0; par < 2; ++par) {
            int vi = 0, ti = 0;
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                // the reads of this slot go to the other set; they are waited for at the top of the next iteration
#pragma unroll
                for (int j = 0; j < NL; ++j)
                    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f[par ^ 1][m]) : "v"(addr), "n"(4096) : "memory");
                if (m == 0) asm volatile("s_waitcnt lgkmcnt(%0)" :: "n"(NL) : "memory");     // everything but this slot's reads has landed
                const bf16x8 a = __builtin_bit_cast(bf16x8, f[par][m]);
                c[m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[m & 3], 0, 0, 0);
#pragma unroll
                for (int j = 0; j < 3; ++j) { x[vi & 15] = __builtin_fmaf(x[vi & 15], fa, fb); ++vi; }
                y[ti & 15] = __builtin_amdgcn_exp2f(y[ti & 15]); ++ti;
            }
        }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    const long long t1 = clock64();
    float s = 0.f;
    for (int i = 0; i < 16; ++i) s += x[i] + y[i];
    for (int j = 0; j < 4; ++j) s += c[j][j];
    for (int i = 0; i < 4; ++i) s += f[0][i][0] + f[1][i][1];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
    if ((threadIdx.x & 63) == 0 && blockIdx.x == 0) {
        atomicMin((unsigned long long *)&cyc[0], (unsigned long long)t0);
        atomicMax((unsigned long long *)&cyc[1], (unsigned long long)t1);
    }
}

template <int NL>
static void run_lds_issue(float *d, long long *dc, const char *name)
{
    const int iters = 4000;
    printf("%-44s", name);
    for (int w = 1; w <= 2; ++w) {
        lds_issue_kernel<NL><<<256, 256 * w>>>(d, dc, iters);
        CHECK(hipDeviceSynchronize());
        long long init[2] = {0x7fffffffffffffffLL, 0};
        CHECK(hipMemcpy(dc, init, 16, hipMemcpyHostToDevice));
        lds_issue_kernel<NL><<<256, 256 * w>>>(d, dc, iters);
        CHECK(hipDeviceSynchronize());
        long long cc[2];
        CHECK(hipMemcpy(cc, dc, 16, hipMemcpyDeviceToHost));
        const double per_slot = (double)(cc[1] - cc[0]) / iters / 4 / w;
        printf("  w%d %5.1f (%3.0f%%)", w, per_slot, 100.0 * 32.0 / per_slot);
    }
    printf("\n");
}

// ---- section 6: data dependence of the sustained matrix rate
__device__ uint32_t mix_u32(uint32_t x) { x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; return x ^ (x >> 16); }
template <int RANDOM, int NV, int NT>
__global__ __launch_bounds__(256) void data_kernel(float *out, int iters)
{
    bf16x8 a[8], b[8];      // eight fragments each; every instruction pairs another two
    for (int j = 0; j < 8; ++j)
        for (int i = 0; i < 8; ++i) {
            const uint32_t h = mix_u32(threadIdx.x * 977u + blockIdx.x * 131u + j * 17u + i);
            a[j][i] = (__bf16)(RANDOM ? ((int)(h & 0xffff) - 32768) * (1.0f / 16384.f) : 1.0f);
            b[j][i] = (__bf16)(RANDOM ? ((int)(h >> 16) - 32768) * (1.0f / 16384.f) : 1.0f);
        }
    f32x16 c[4];
    for (int j = 0; j < 4; ++j) for (int i = 0; i < 16; ++i) c[j][i] = 0.f;
    float x[16], y[16];     // independent chains of fma and of exp2 (kept bounded)
    for (int i = 0; i < 16; ++i) { x[i] = threadIdx.x * 1e-3f + i; y[i] = threadIdx.x * 1e-4f + i * 0.01f; }
    const float fa = 1.0001f, fb = 1e-4f;
    for (int it = 0; it < iters; it += 8) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            int vi = 0, ti = 0;
#pragma unroll
            for (int m = 0; m < 8; ++m) {
                c[m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[m], b[(m + r) & 7], c[m & 3], 0, 0, 0);
#pragma unroll
                for (int j = 0; j < NV; ++j) { x[vi & 15] = __builtin_fmaf(x[vi & 15], fa, fb); ++vi; }
#pragma unroll
                for (int j = 0; j < NT; ++j) { y[ti & 15] = __builtin_amdgcn_exp2f(y[ti & 15] * 0.5f - 1.0f); ++ti; }
            }
        }
    }
    float s = 0.f;
    for (int j = 0; j < 4; ++j) for (int i = 0; i < 16; ++i) s += c[j][i];
    for (int i = 0; i < 16; ++i) s += x[i] + y[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <int RANDOM, int NV = 0, int NT = 0>
static void run_data(float *d, const char *name)
{
    const int iters = 40000;        // x 8 instructions x 32 cycles x 2 wavefronts per SIMD: about 10 ms
    data_kernel<RANDOM, NV, NT><<<512, 256>>>(d, 1000);
    CHECK(hipDeviceSynchronize());
    const auto w0 = std::chrono::steady_clock::now();
    data_kernel<RANDOM, NV, NT><<<512, 256>>>(d, iters);
    CHECK(hipDeviceSynchronize());
    const double us = std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - w0).count();
    const double flops = 512.0 * 4 * iters * 8 * 32768.0;
    printf("%-44s  %6.2f ms  %5.0f TFLOP/s  (= %4.2f GHz at 32 cycles per instruction)\n", name, us / 1e3, flops / (us * 1e-6) / 1e12,
           flops / (us * 1e-6) / (256.0 * 4 * 1024.0) / 1e9);
}

// ---- section 4: LDS fragment reads
template <int MODE, int D>
__device__ int chunk_off(int r, int c)
{
    constexpr int CPR = D / 8;
    int f;
    if (MODE == 0) f = r & 7;
    else f = D == 64 ? (r & 7) : (((r & 3) << 2) | ((r >> 2) & 3));
    return r * (D * 2) + ((c ^ f) & (CPR - 1)) * 16;
}

template <int MODE, int D, int KIND>
__global__ __launch_bounds__(256) void lds_kernel(float *out, int iters)
{
    __shared__ __attribute__((aligned(1024))) char smem[64 * 1024];
    const int tid = threadIdx.x, lane = tid & 63, lq = lane & 31, hh = lane >> 5;
    for (int i = tid; i < 64 * 1024 / 4; i += 256) reinterpret_cast<float *>(smem)[i] = (float)i;
    __syncthreads();
    int off[4];
    if (KIND == 0) {
        for (int kb = 0; kb < 4; ++kb) off[kb] = chunk_off<MODE, D>(lq, 2 * kb + hh);
    } else {
        const int grp = lane >> 4, h2 = grp >> 1, nh = grp & 1, s = lane & 15, row = 4 * h2 + (s >> 2);
        for (int db = 0; db < 4; ++db) off[db] = chunk_off<MODE, D>(row, 4 * (db & (D / 32 - 1)) + 2 * nh + ((s & 3) >> 1)) + (s & 1) * 8;
    }
    f32x4 acc = {0, 0, 0, 0};
    for (int it = 0; it < iters; ++it) {
        const char *base = smem + (it & 3) * 8192;
        if (KIND == 0) {
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) acc += *reinterpret_cast<const f32x4 *>(base + off[kb]);
        } else {
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                const int hi = (MODE == 1 && D == 128) ? (off[db] ^ 32) : off[db];
                const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(base + off[db]));
                const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(base + hi + 8 * D * 2));
                acc[0] += (float)a[0];
                acc[1] += (float)b[1];
            }
        }
    }
    out[blockIdx.x * 256 + tid] = acc[0] + acc[1] + acc[2] + acc[3];
}

template <int MODE, int D, int KIND>
static void run_lds(float *d, const char *name)
{
    const int iters = 20000;
    printf("%-44s", name);
    for (int wg = 1; wg <= 2; ++wg) {     // workgroups of four wavefronts per compute unit
        hipEvent_t e0, e1;
        CHECK(hipEventCreate(&e0));
        CHECK(hipEventCreate(&e1));
        lds_kernel<MODE, D, KIND><<<256 * wg, 256>>>(d, 100);
        CHECK(hipDeviceSynchronize());
        CHECK(hipEventRecord(e0));
        lds_kernel<MODE, D, KIND><<<256 * wg, 256>>>(d, iters);
        CHECK(hipEventRecord(e1));
        CHECK(hipDeviceSynchronize());
        float ms;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        const double instr_per_cu = (double)iters * (KIND == 0 ? 4 : 8) * 4 * wg;
        printf("  %d wg/CU: %5.2f ns per wave-instruction per CU", wg, ms * 1e6 / instr_per_cu);
        CHECK(hipEventDestroy(e0));
        CHECK(hipEventDestroy(e1));
    }
    printf("\n");
}

int main()
{
    float *d;
    long long *dc;
    CHECK(hipMalloc(&d, 512 * 1024 * 4));
    CHECK(hipMalloc(&dc, 16));
    printf("# 1-3. SIMD cycles per slot of one wavefront (slot = one matrix instruction and the work listed with it, or that work alone);\n"
           "#      wN = N wavefronts per SIMD; (matrix pipe busy = 32 cycles / slot)\n");
    run_issue<1, 0, 0, 0>(d, dc, "mfma alone");
    run_issue<0, 4, 0, 0>(d, dc, "4 fma");
    run_issue<0, 0, 4, 0>(d, dc, "4 exp2");
    run_issue<1, 2, 0, 0>(d, dc, "mfma + 2 fma");
    run_issue<1, 4, 0, 0>(d, dc, "mfma + 4 fma");
    run_issue<1, 6, 0, 0>(d, dc, "mfma + 6 fma");
    run_issue<1, 8, 0, 0>(d, dc, "mfma + 8 fma");
    run_issue<1, 0, 2, 0>(d, dc, "mfma + 2 exp2");
    run_issue<1, 3, 1, 0>(d, dc, "mfma + 3 fma + 1 exp2 (backward's mix)");
    run_issue<1, 6, 2, 0>(d, dc, "mfma + 6 fma + 2 exp2 (forward's mix, d=64)");
    run_issue<1, 3, 1, 2>(d, dc, "mfma + 3 fma + 1 exp2 + 4 scalar");
    run_issue<1, 3, 1, 4>(d, dc, "mfma + 3 fma + 1 exp2 + 8 scalar");
    run_issue<1, 3, 1, 8>(d, dc, "mfma + 3 fma + 1 exp2 + 16 scalar");
    printf("# 5. as 3., operands of the matrix instructions read from LDS one iteration ahead (ds_read_b128 per matrix instruction)\n");
    run_lds_issue<0>(d, dc, "mfma + 3 fma + 1 exp2, no LDS read");
    run_lds_issue<1>(d, dc, "mfma + 3 fma + 1 exp2 + 1 ds_read_b128");
    printf("# 6. a loop of matrix instructions, two wavefronts per SIMD, wall time of a 10 ms launch (clock included)\n");
    run_data<0>(d, "constant operands (all ones)");
    run_data<1>(d, "random operands in [-2, 2)");
    run_data<1, 3, 1>(d, "random, + 3 fma + 1 exp2 per instruction");
    run_data<1, 6, 2>(d, "random, + 6 fma + 2 exp2 per instruction");
    run_data<0>(d, "constant operands (all ones), again");
    run_data<1>(d, "random operands in [-2, 2), again");
    run_data<1, 3, 1>(d, "random, + 3 fma + 1 exp2, again");
    run_data<1, 6, 2>(d, "random, + 6 fma + 2 exp2, again");
    printf("# 4. LDS fragment reads, [rows][D] bf16 tiles, time per wave-instruction per compute unit\n");
    run_lds<0, 64, 0>(d, "ds_read_b128 by rows, D=64, r&7");
    run_lds<0, 128, 0>(d, "ds_read_b128 by rows, D=128, r&7");
    run_lds<1, 128, 0>(d, "ds_read_b128 by rows, D=128, tile_swizzle");
    run_lds<0, 64, 1>(d, "ds_read_b64_tr_b16, D=64, r&7");
    run_lds<0, 128, 1>(d, "ds_read_b64_tr_b16, D=128, r&7");
    run_lds<1, 128, 1>(d, "ds_read_b64_tr_b16, D=128, tile_swizzle");
    return 0;
}
