// Host-side launchers of the segment-attention kernels; called by the C ABI only.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace lss {

typedef __bf16 bf16_t;

// One segment's problem, as the kernels see it (Eq. 2 of Section 3; device pointers).
struct SegShape {
    int64_t s0;      // global index of the segment's first query row
    int l_s, l_x;    // query rows of the segment, key/value rows of the sequence
    int B, H, d;
    int causal;
    int skip_tail;   // causal backward: leave key tiles that no query of the segment sees unwritten (not zero-filled)
};

// Dropout on the attention weights (Section 2.2); thr == 0 means none.  A weight is kept when its
// 32-bit random number (lss_common.h: drop_keep) is >= thr; kept weights are multiplied by
// scale = 1 / (1 - p).
struct DropArgs {
    uint32_t thr;
    float scale;
    uint32_t seed_lo, seed_hi;
};

// How many key ranges ("splits") a query tile's keys are divided into so that a
// skinny segment (l_s << l_x) still fills the chip.  Shape-only, deterministic.
// `rows_per_wg` is the query-tile height of the kernel that will run (it differs per dtype).
int choose_splits(int l_s, int l_x, int B, int H, int rows_per_wg);
// Forward: the largest split count the workspace is sized for (shape-only), and the count a launch
// uses for the `kv_tiles` 64-key tiles its query tiles actually see (never above the former).
int max_fwd_splits(int l_s, int l_x, int B, int H, int rows_per_wg);
int pick_fwd_splits(int l_s, int B, int H, int rows_per_wg, int64_t kv_tiles, int max_splits, int resident);
int fwd_wgs_per_cu(int elem_bytes, int d);      // forward workgroups a compute unit holds at once ("resident")
int fwd_rows_per_wg(int elem_bytes, int d);     // query rows per workgroup of the forward kernel
int dq_rows_per_wg(int elem_bytes, int d);      // ... and of the dQ kernel

struct Workspace {
    // forward
    float *o_part;    // [splits, B*H, l_s, d] in the storage type (bf16 kernels write bf16 here)
    float *lse_part;  // [splits, B*H, l_s]
    // backward
    float *D;         // [B*H, l_s]      rowsum(dO * out)   (bf16 kernels: its negative)
    float *Ls;        // [B*H, l_s]      bf16 kernels: -lse * sqrt(d), start value of the S accumulators
    float *dq_part;   // [splits, B, l_s, H, d]
    uint32_t *row_key; // [B*H, l_s]      dropout in the bf16 dK/dV workgroups: the generator's key of every query row
};
size_t workspace_bytes(int l_s, int l_x, int B, int H, int d, int elem_bytes);
size_t bwd_workspace_bytes(int l_s, int l_x, int B, int H, int d, int elem_bytes);    // the leading part a backward call uses
Workspace carve_workspace(void *base, int l_s, int l_x, int B, int H, int d, int elem_bytes);

template <typename T>
hipError_t launch_fwd(const SegShape &s, const DropArgs &drop, const T *q, const T *k, const T *v, T *out, float *lse,
                      const Workspace &ws, hipStream_t st);

template <typename T>
hipError_t launch_bwd(const SegShape &s, const DropArgs &drop, const T *q, const T *k, const T *v, const T *out,
                      const float *lse, const T *dO, T *dq, float *dk_part, float *dv_part,
                      const Workspace &ws, hipStream_t st);

// tuned bf16 kernels (lss_fwd_bf16.hip)
int fwd_bf16_rows_per_workgroup(int d);
hipError_t launch_fwd_bf16_main(const SegShape &s, const DropArgs &drop, const bf16_t *q, const bf16_t *k,
                                const bf16_t *v, bf16_t *out, float *lse, const Workspace &ws, int n_splits, hipStream_t st);

// tuned bf16 kernels (lss_bwd_bf16.hip): dQ kernel (also writes D = rowsum(dO * out)) then dK/dV kernel
int dq_bf16_rows_per_workgroup(int d);
hipError_t launch_bwd_bf16_main(const SegShape &s, const DropArgs &drop, const bf16_t *q, const bf16_t *k,
                                const bf16_t *v, const bf16_t *out, const float *lse, const bf16_t *dO, bf16_t *dq,
                                float *dk_part, float *dv_part, const Workspace &ws, int n_splits, hipStream_t st);

// Optional per-kernel timing for benchmarks (lss_timing.h): when enabled, every launch site
// brackets its kernel with a pair of HIP events on the launch stream.  One id per __global__
// function (per role where several entry points share one).
enum KernelId { K_FWD = 0, K_FWD_MERGE, K_ROWDOT, K_DQ, K_DQ_MERGE, K_DKV, K_REDUCE, K_BWD_MAIN_BF16, K_PROJ_FWD, K_PROJ_BWD,
                K_PE_FWD, K_PE_BWD, K_LN_FWD, K_LN_BWD, K_LN_PARAMS, K_GELU_FWD, K_GELU_BWD, K_LINEAR_FWD, K_LINEAR_BWD, K_RESIDUAL, K_LINEAR_WGRAD,
                K_FWD_BF16, K_BWD_PREP_BF16, K_COUNT };
void timing_begin(int id, hipStream_t st);
void timing_end(int id, hipStream_t st);
struct TimedLaunch {    // RAII bracket around one kernel launch
    int id; hipStream_t st;
    TimedLaunch(int id_, hipStream_t st_) : id(id_), st(st_) { timing_begin(id, st); }
    ~TimedLaunch() { timing_end(id, st); }
};

constexpr int kMaxReduceParts = 64;
hipError_t launch_reduce(const float *const *parts, int n, const int64_t *rows_valid, int64_t l_x,
                         int64_t B, int64_t H, int64_t d, float *out, hipStream_t st);

// the linear maps around the attention (lss_proj.hip); E = H * d, a multiple of 128
hipError_t launch_project_qkv(const bf16_t *x, const bf16_t *w_q, const bf16_t *w_kv, int64_t s0, int l_s, int l_x,
                              int B, int E, bf16_t *q_seg, bf16_t *k, bf16_t *v, hipStream_t st);
hipError_t launch_project_bwd(const bf16_t *dq, const float *dk_part, const float *dv_part, const bf16_t *w_q,
                              const bf16_t *w_kv, int l_s, int l_x, int rows_valid, int B, int E, int skip_tail,
                              float *dx_q, float *dx_part, hipStream_t st);


// general bf16 linear maps with the same GEMM kernel (the feed-forward unit's two transforms):
// c[rows, N] = a[rows, K] w[K, N]   and   da[rows, K] = dc[rows, N] w[K, N]^T;  K, N multiples of 128
// with gelu_c: also gelu_c[rows, N] = GeLU(c);  with gelu_u [rows, K]: da = (dc w^T) * GeLU'(gelu_u)
hipError_t launch_linear_fwd(const bf16_t *a, const bf16_t *w, int rows, int K, int N, bf16_t *c, bf16_t *gelu_c,
                             hipStream_t st);
hipError_t launch_linear_bwd_input(const bf16_t *dc, const bf16_t *w, const bf16_t *gelu_u, int rows, int K, int N,
                                   bf16_t *da, hipStream_t st);

// dw[K, N] (float) = a[rows, K]^T dc[rows, N]; rows >= 1; scratch of linear_bwd_weight_scratch_bytes() bytes
size_t linear_bwd_weight_scratch_bytes(int rows, int K, int N);
hipError_t launch_linear_bwd_weight(const bf16_t *a, const bf16_t *dc, int rows, int K, int N, float *dw, float *scratch,
                                    hipStream_t st);

// one segment's share of the projection weights' gradients: dw_q [E][E], dw_kv [E][2E] (float)
size_t project_bwd_weight_scratch_bytes(int l_s, int l_x, int B, int E);        // for any rows_valid <= l_x
size_t project_bwd_weight_scratch_needed(int l_s, int rows_valid, int B, int E); // what one call uses
hipError_t launch_project_bwd_weight(const bf16_t *x, const bf16_t *dq, const float *dk_part, const float *dv_part, int64_t s0,
                                     int l_s, int l_x, int rows_valid, int B, int E, float *dw_q, float *dw_kv, float *scratch,
                                     hipStream_t st);

// segment-local row operations (lss_rows.hip); E a multiple of 8
hipError_t launch_embed_pe_fwd(const bf16_t *tok, const bf16_t *pe, int64_t s0, int l_s, int B, int E, bf16_t *x,
                               hipStream_t st);
hipError_t launch_embed_pe_bwd(const bf16_t *dx, int l_s, int B, int E, float *dpe, hipStream_t st);
hipError_t launch_residual_add(const bf16_t *x, const bf16_t *delta, const DropArgs &drop, int64_t s0, int l_s, int B, int E,
                               bf16_t *out, hipStream_t st);
int layernorm_max_columns();
size_t layernorm_bwd_scratch_bytes(int64_t rows, int E);
hipError_t launch_layernorm_fwd(const bf16_t *x, const float *gamma, const float *beta, float eps, int64_t rows, int E,
                                bf16_t *y, float *mean, float *rstd, hipStream_t st);
hipError_t launch_layernorm_bwd(const bf16_t *x, const float *gamma, const float *mean, const float *rstd, const bf16_t *dy,
                                int64_t rows, int E, bf16_t *dx, float *dgamma, float *dbeta, float *scratch, hipStream_t st);
hipError_t launch_gelu_fwd(const bf16_t *u, int64_t n, bf16_t *g, hipStream_t st);
hipError_t launch_gelu_bwd(const bf16_t *u, const bf16_t *dg, int64_t n, bf16_t *du, hipStream_t st);

} // namespace lss
