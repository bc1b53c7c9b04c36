// C ABI of the segment-attention library: argument checks, workspace, dispatch.
// Every entry point is documented in include/lss_attn.h.
#include "lss_attn.h"
#include "lss_common.h"
#include "lss_kernels.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <atomic>
#include <initializer_list>
#include <mutex>

namespace lss {

int fwd_rows_per_wg(int elem_bytes, int d) { return elem_bytes == 2 ? fwd_bf16_rows_per_workgroup(d) : 128; }
int dq_rows_per_wg(int elem_bytes, int d) { return elem_bytes == 2 ? dq_bf16_rows_per_workgroup(d) : 128; }

int choose_splits(int l_s, int l_x, int B, int H, int rows_per_wg)
{
    // aim for >= 2 workgroups per compute unit (256 of them); a split needs >= 4 key tiles
    const int64_t wgs = (int64_t)((l_s + rows_per_wg - 1) / rows_per_wg) * B * H;
    if (wgs <= 0) return 1;
    int64_t want = (512 + wgs - 1) / wgs;
    const int64_t tiles = (l_x + 63) / 64;
    if (want > tiles / 4) want = tiles / 4;
    if (want > 16) want = 16;
    if (want < 1) want = 1;
    return (int)want;
}

int max_fwd_splits(int l_s, int l_x, int B, int H, int rows_per_wg)
{
    // up to four workgroups per compute unit; a split needs >= 4 key tiles
    const int64_t wgs = (int64_t)((l_s + rows_per_wg - 1) / rows_per_wg) * B * H;
    if (wgs <= 0) return 1;
    int64_t most = (1024 + wgs - 1) / wgs;
    const int64_t tiles = (l_x + 63) / 64;
    if (most > tiles / 4) most = tiles / 4;
    if (most > 16) most = 16;
    return most < 1 ? 1 : (int)most;
}

int fwd_wgs_per_cu(int elem_bytes, int d) { return elem_bytes == 2 ? (d == 64 ? 3 : 1) : 2; }

int pick_fwd_splits(int l_s, int B, int H, int rows_per_wg, int64_t kv_tiles, int max_splits, int resident)
{
    // Measured on the bf16 forward kernels (8..2048 query tiles, 1..16 splits), in units of the time a
    // lone workgroup takes per 64-key tile (0.77 us at d = 64): a launch takes about
    //   (key tiles per workgroup + 8) x g(n) + 6 if split,   n = workgroups per compute unit, rounded up,
    // 8 for a workgroup's start and results, 6 for the merge launch, g(1) = 1 and g(n) = 0.17 + 0.65 n
    // where several workgroups share a compute unit (a second co-resident workgroup adds about a
    // third of a workgroup's throughput), g(n) = n where only one fits.  What matters most is
    // that the workgroup count lands just below a multiple of the 256 compute units.  The smallest
    // count within 3 % of the best estimate is taken.
    const int64_t wgs = (int64_t)((l_s + rows_per_wg - 1) / rows_per_wg) * B * H;
    if (wgs <= 0 || max_splits <= 1) return 1;
    double best = 0.0;
    int best_s = 1;
    for (int sp = 1; sp <= max_splits; ++sp) {
        if (sp > 1 && kv_tiles / sp < 8) break;        // shorter splits cost more than they gain
        const int64_t per_cu = (wgs * sp + 255) / 256;
        const double g = per_cu <= 1 ? 1.0 : resident <= 1 ? (double)per_cu : 0.17 + 0.65 * (double)per_cu;
        const double t = ((double)((kv_tiles + sp - 1) / sp) + 8.0) * g + (sp > 1 ? 6.0 : 0.0);
        if (sp == 1 || t < 0.97 * best) { best = t; best_s = sp; }
    }
    return best_s;
}

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// The backward's regions come first: a backward call needs only the first `bwd_total` bytes.
struct WsLayout { size_t D, Ls, dq_part, row_key, bwd_total, o_part, lse_part, total; };
static WsLayout ws_layout(int l_s, int l_x, int B, int H, int d, int elem_bytes)
{
    // forward and dQ kernels may use different tile heights, hence different split counts
    const size_t sp_f = (size_t)max_fwd_splits(l_s, l_x, B, H, fwd_rows_per_wg(elem_bytes, d));
    const size_t sp_q = (size_t)choose_splits(l_s, l_x, B, H, dq_rows_per_wg(elem_bytes, d));
    const size_t rows = (size_t)B * H * l_s;
    WsLayout w;
    size_t off = 0;
    w.D = off;        off += align256(rows * sizeof(float));
    w.Ls = off;       off += align256(rows * sizeof(float));
    w.dq_part = off;  off += align256(sp_q > 1 ? sp_q * rows * d * sizeof(float) : 0);
    w.row_key = off;  off += align256(rows * sizeof(uint32_t));
    w.bwd_total = off;
    w.o_part = off;   off += align256(sp_f > 1 ? sp_f * rows * d * (size_t)elem_bytes : 0);     // in the storage type
    w.lse_part = off; off += align256(sp_f > 1 ? sp_f * rows * sizeof(float) : 0);
    w.total = off;
    return w;
}
size_t workspace_bytes(int l_s, int l_x, int B, int H, int d, int elem_bytes)
{
    return ws_layout(l_s, l_x, B, H, d, elem_bytes).total;
}
size_t bwd_workspace_bytes(int l_s, int l_x, int B, int H, int d, int elem_bytes)
{
    return ws_layout(l_s, l_x, B, H, d, elem_bytes).bwd_total;
}
Workspace carve_workspace(void *base, int l_s, int l_x, int B, int H, int d, int elem_bytes)
{
    const WsLayout w = ws_layout(l_s, l_x, B, H, d, elem_bytes);
    char *p = static_cast<char *>(base);
    Workspace ws;
    ws.o_part = reinterpret_cast<float *>(p + w.o_part);
    ws.lse_part = reinterpret_cast<float *>(p + w.lse_part);
    ws.D = reinterpret_cast<float *>(p + w.D);
    ws.Ls = reinterpret_cast<float *>(p + w.Ls);
    ws.dq_part = reinterpret_cast<float *>(p + w.dq_part);
    ws.row_key = reinterpret_cast<uint32_t *>(p + w.row_key);
    return ws;
}

} // namespace lss

namespace {

thread_local char g_err[256] = "";
// the scratch buffer registered for each GPU (lss_set_workspace), indexed by HIP device id
constexpr int kMaxDevices = 64;
std::mutex g_ws_mutex;
void *g_ws_ptr[kMaxDevices] = {};
size_t g_ws_bytes[kMaxDevices] = {};

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

int check_shape(int64_t s0, int64_t l_s, int64_t l_x, int64_t B, int64_t H, int64_t d)
{
    if (d != 64 && d != 128) return fail(LSS_ERR_UNSUPPORTED_D, "d = %lld: only 64 and 128 are supported", (long long)d);
    if (l_s < 0 || B < 0 || H < 1 || l_x < 1) return fail(LSS_ERR_SHAPE, "bad shape: l_s=%lld l_x=%lld B=%lld H=%lld", (long long)l_s, (long long)l_x, (long long)B, (long long)H);
    if (B * H > 65535) return fail(LSS_ERR_SHAPE, "B*H = %lld exceeds 65535", (long long)(B * H));
    if (l_x > (int64_t)1 << 30) return fail(LSS_ERR_SHAPE, "l_x = %lld exceeds 2^30", (long long)l_x);
    if (s0 < 0 || s0 + l_s > l_x) return fail(LSS_ERR_RANGE, "segment [%lld, %lld) is outside [0, %lld)", (long long)s0, (long long)(s0 + l_s), (long long)l_x);
    return LSS_OK;
}

// the kernels' dropout arguments from the probability and the seed (p already checked to be in [0, 1))
lss::DropArgs dropout_args(double p, uint64_t seed)
{
    const double t = std::floor(p * 4294967296.0 + 0.5);
    lss::DropArgs a;
    a.thr = t >= 4294967295.0 ? 4294967295u : (t <= 0.0 ? 0u : (uint32_t)t);
    a.scale = (float)(1.0 / (1.0 - p));
    a.seed_lo = (uint32_t)seed;
    a.seed_hi = (uint32_t)(seed >> 32);
    return a;
}
int check_dropout(double p)
{
    if (!(p >= 0.0 && p < 1.0)) return fail(LSS_ERR_RANGE, "dropout probability %g is outside [0, 1)", p);
    return LSS_OK;
}

int current_device(int *dev)
{
    if (hipGetDevice(dev) != hipSuccess) {      // a host without a GPU: argument checks still work, against slot 0
        (void)hipGetLastError();
        *dev = 0;
    }
    if (*dev < 0 || *dev >= kMaxDevices) return fail(LSS_ERR_WORKSPACE, "device id %d is not below %d", *dev, kMaxDevices);
    return LSS_OK;
}

// The scratch of one call: the caller's own buffer (`own`, `own_bytes`) if given, else the one
// registered for the current GPU.
// `bwd_only`: the buffer need only hold the backward's regions (the built-in scratch of
// lss_segment_attn_bwd_noalloc); the forward's pointers then lie outside it and are never used.
int get_workspace(int l_s, int l_x, int B, int H, int d, int elem_bytes, void *own, size_t own_bytes, lss::Workspace *ws,
                  bool bwd_only = false)
{
    const size_t need = bwd_only ? lss::bwd_workspace_bytes(l_s, l_x, B, H, d, elem_bytes)
                                 : lss::workspace_bytes(l_s, l_x, B, H, d, elem_bytes);
    void *base = own;
    size_t have = own_bytes;
    if (own == nullptr) {
        int dev = 0;
        if (int rc = current_device(&dev)) return rc;
        std::lock_guard<std::mutex> lock(g_ws_mutex);
        base = g_ws_ptr[dev];
        have = g_ws_bytes[dev];
    }
    if (need > 0 && (base == nullptr || have < need))
        return fail(LSS_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu %s", need, base ? have : (size_t)0,
                    own ? "passed" : "registered for this GPU (lss_set_workspace)");
    *ws = lss::carve_workspace(base, l_s, l_x, B, H, d, elem_bytes);
    if (bwd_only) ws->o_part = ws->lse_part = nullptr;
    return LSS_OK;
}

// ---- built-in scratch of lss_segment_attn_bwd_noalloc
// Device memory that exists from the moment the library's code object is loaded on a GPU until the
// process ends; each GPU holds its own copy at its own address.  In host code the array's name is only
// a handle for hipGetSymbolAddress: kernels are always given the address that call returned.
static __device__ __align__(256) unsigned char scratch[LSS_NOALLOC_SCRATCH_BYTES];
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

int builtin_scratch(void **ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return fail(LSS_ERR_WORKSPACE, "built-in scratch: no current GPU (or its device id is not below %d)", kMaxDevices);
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {        // first call on this GPU, which is current
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || p == nullptr) {
            (void)hipGetLastError();
            return fail(LSS_ERR_WORKSPACE, "built-in scratch: hipGetSymbolAddress failed on device %d: %s", dev, hipGetErrorString(e));
        }
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return LSS_OK;
}

int check_flags(unsigned flags)
{
    if (flags & ~LSS_FLAG_SKIP_MASKED_TAIL) return fail(LSS_ERR_RANGE, "unknown flag bits 0x%x", flags & ~LSS_FLAG_SKIP_MASKED_TAIL);
    return LSS_OK;
}

template <typename T>
int fwd_impl(const void *q, const void *k, const void *v, int64_t s0, int64_t l_s, int64_t l_x, int64_t B,
             int64_t H, int64_t d, int causal, double p_drop, uint64_t seed, unsigned flags, void *wsp, size_t wsp_bytes,
             void *out, float *lse, void *stream)
{
    if (int rc = check_shape(s0, l_s, l_x, B, H, d)) return rc;
    if (int rc = check_dropout(p_drop)) return rc;
    if (int rc = check_flags(flags)) return rc;
    if (misaligned(wsp)) return fail(LSS_ERR_ALIGN, "forward: workspace must be 16-byte aligned");
    if (l_s == 0 || B == 0) return LSS_OK;
    if (!q || !k || !v || !out || !lse) return fail(LSS_ERR_NULL, "forward: NULL tensor pointer");
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out) || misaligned(lse))
        return fail(LSS_ERR_ALIGN, "forward: tensor pointers must be 16-byte aligned");
    lss::Workspace ws;
    if (int rc = get_workspace((int)l_s, (int)l_x, (int)B, (int)H, (int)d, (int)sizeof(T), wsp, wsp_bytes, &ws)) return rc;
    const lss::SegShape s{s0, (int)l_s, (int)l_x, (int)B, (int)H, (int)d, causal ? 1 : 0, 0};
    const lss::DropArgs drop = dropout_args(p_drop, seed);
    const hipError_t e = lss::launch_fwd<T>(s, drop, static_cast<const T *>(q), static_cast<const T *>(k),
                                            static_cast<const T *>(v), static_cast<T *>(out), lse, ws,
                                            static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(LSS_ERR_LAUNCH, "forward launch failed: %s", hipGetErrorString(e));
    return LSS_OK;
}

template <typename T>
int bwd_impl(const void *q, const void *k, const void *v, int64_t s0, int64_t l_s, int64_t l_x, int64_t B,
             int64_t H, int64_t d, int causal, double p_drop, uint64_t seed, unsigned flags, void *wsp, size_t wsp_bytes,
             const void *out, const float *lse, const void *dO, void *dq, float *dk_part, float *dv_part, void *stream,
             bool bwd_only_scratch = false)
{
    if (int rc = check_shape(s0, l_s, l_x, B, H, d)) return rc;
    if (int rc = check_dropout(p_drop)) return rc;
    if (int rc = check_flags(flags)) return rc;
    if (misaligned(wsp)) return fail(LSS_ERR_ALIGN, "backward: workspace must be 16-byte aligned");
    if (B == 0) return LSS_OK;
    if (!k || !v || !dk_part || !dv_part) return fail(LSS_ERR_NULL, "backward: NULL tensor pointer");
    if (l_s > 0 && (!q || !out || !lse || !dO || !dq)) return fail(LSS_ERR_NULL, "backward: NULL tensor pointer");
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out) || misaligned(lse) || misaligned(dO) ||
        misaligned(dq) || misaligned(dk_part) || misaligned(dv_part))
        return fail(LSS_ERR_ALIGN, "backward: tensor pointers must be 16-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (l_s == 0) {     // an empty segment contributes nothing: the partials are all zero
        // Written by the sum kernel over one part with no valid rows (it reads nothing then):
        // a kernel launch, not a memset, so that a caller may record the call into a graph.
        const int64_t none = 0;
        for (float *part : {dk_part, dv_part}) {
            const float *src = part;
            const hipError_t e = lss::launch_reduce(&src, 1, &none, l_x, B, H, d, part, st);
            if (e != hipSuccess) return fail(LSS_ERR_LAUNCH, "backward zero fill failed: %s", hipGetErrorString(e));
        }
        return LSS_OK;
    }
    lss::Workspace ws;
    if (int rc = get_workspace((int)l_s, (int)l_x, (int)B, (int)H, (int)d, (int)sizeof(T), wsp, wsp_bytes, &ws, bwd_only_scratch))
        return rc;
    const lss::SegShape s{s0, (int)l_s, (int)l_x, (int)B, (int)H, (int)d, causal ? 1 : 0,
                          (flags & LSS_FLAG_SKIP_MASKED_TAIL) ? 1 : 0};
    const lss::DropArgs drop = dropout_args(p_drop, seed);
    const hipError_t e = lss::launch_bwd<T>(s, drop, static_cast<const T *>(q), static_cast<const T *>(k),
                                            static_cast<const T *>(v), static_cast<const T *>(out), lse,
                                            static_cast<const T *>(dO), static_cast<T *>(dq), dk_part, dv_part, ws, st);
    if (e != hipSuccess) return fail(LSS_ERR_LAUNCH, "backward launch failed: %s", hipGetErrorString(e));
    return LSS_OK;
}

} // namespace

extern "C" {

int lss_version(void) { return 100; }

const char *lss_last_error(void) { return g_err; }

size_t lss_workspace_bytes(int64_t l_s, int64_t l_x, int64_t B, int64_t H, int64_t d, int elem_bytes)
{
    if ((elem_bytes != 2 && elem_bytes != 4) || (d != 64 && d != 128)) return 0;
    if (l_s <= 0 || l_x < 1 || B <= 0 || H < 1 || l_s > l_x || l_x > (int64_t)1 << 30 || B * H > 65535) return 0;
    return lss::workspace_bytes((int)l_s, (int)l_x, (int)B, (int)H, (int)d, elem_bytes);
}

int lss_set_workspace(void *device_ptr, size_t bytes)
{
    if (device_ptr == nullptr && bytes != 0) return fail(LSS_ERR_NULL, "workspace pointer is NULL but bytes = %zu", bytes);
    if (misaligned(device_ptr)) return fail(LSS_ERR_ALIGN, "workspace must be 16-byte aligned");
    int dev = 0;
    if (int rc = current_device(&dev)) return rc;
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    g_ws_ptr[dev] = device_ptr;
    g_ws_bytes[dev] = device_ptr ? bytes : 0;
    return LSS_OK;
}

int lss_segment_attn_fwd(const void *q_seg, const void *k, const void *v, int64_t seg_offset, int64_t l_s,
                         int64_t l_x, int64_t B, int64_t H, int64_t d, int causal, void *out, float *lse,
                         void *stream)
{
    return fwd_impl<lss::bf16_t>(q_seg, k, v, seg_offset, l_s, l_x, B, H, d, causal, 0.0, 0, 0u, nullptr, 0, out, lse, stream);
}

int lss_segment_attn_bwd(const void *q_seg, const void *k, const void *v, int64_t seg_offset, int64_t l_s,
                         int64_t l_x, int64_t B, int64_t H, int64_t d, int causal, const void *out,
                         const float *lse, const void *dO, void *dq, float *dk_partial, float *dv_partial,
                         void *stream)
{
    return bwd_impl<lss::bf16_t>(q_seg, k, v, seg_offset, l_s, l_x, B, H, d, causal, 0.0, 0, 0u, nullptr, 0, out, lse, dO, dq,
                                 dk_partial, dv_partial, stream);
}

int lss_segment_attn_bwd_noalloc(const void *q_seg, const void *k, const void *v, int64_t seg_offset, int64_t l_s,
                                 int64_t l_x, int64_t B, int64_t H, int64_t d, int causal, const void *out,
                                 const float *lse, const void *dO, void *dq, float *dk_partial, float *dv_partial,
                                 void *stream)
{
    if (int rc = check_shape(seg_offset, l_s, l_x, B, H, d)) return rc;
    const size_t need = (l_s > 0 && B > 0) ? lss::bwd_workspace_bytes((int)l_s, (int)l_x, (int)B, (int)H, (int)d, 2) : 0;
    if (need > (size_t)LSS_NOALLOC_SCRATCH_BYTES)
        return fail(LSS_ERR_WORKSPACE, "the backward of this shape needs %zu bytes of scratch, the built-in buffer holds %zu: use lss_segment_attn_bwd",
                    need, (size_t)LSS_NOALLOC_SCRATCH_BYTES);
    void *ws = nullptr;
    if (need > 0)
        if (int rc = builtin_scratch(&ws)) return rc;
    return bwd_impl<lss::bf16_t>(q_seg, k, v, seg_offset, l_s, l_x, B, H, d, causal, 0.0, 0, 0u, ws,
                                 ws ? (size_t)LSS_NOALLOC_SCRATCH_BYTES : 0, out, lse, dO, dq, dk_partial, dv_partial, stream,
                                 /*bwd_only_scratch=*/true);
}

int lss_segment_attn_fwd_f32(const void *q_seg, const void *k, const void *v, int64_t seg_offset, int64_t l_s,
                             int64_t l_x, int64_t B, int64_t H, int64_t d, int causal, void *out, float *lse,
                             void *stream)
{
    return fwd_impl<float>(q_seg, k, v, seg_offset, l_s, l_x, B, H, d, causal, 0.0, 0, 0u, nullptr, 0, out, lse, stream);
}

int lss_segment_attn_bwd_f32(const void *q_seg, const void *k, const void *v, int64_t seg_offset, int64_t l_s,
                             int64_t l_x, int64_t B, int64_t H, int64_t d, int causal, const void *out,
                             const float *lse, const void *dO, void *dq, float *dk_partial, float *dv_partial,
                             void *stream)
{
    return bwd_impl<float>(q_seg, k, v, seg_offset, l_s, l_x, B, H, d, causal, 0.0, 0, 0u, nullptr, 0, out, lse, dO, dq, dk_partial,
                           dv_partial, stream);
}

int lss_segment_attn_fwd_ex(const void *q_seg, const void *k, const void *v, int64_t seg_offset, int64_t l_s, int64_t l_x,
                            int64_t B, int64_t H, int64_t d, int causal, double p_drop, uint64_t seed, int elem_bytes,
                            unsigned flags, void *workspace, size_t workspace_bytes, void *out, float *lse, void *stream)
{
    if (elem_bytes == 2)
        return fwd_impl<lss::bf16_t>(q_seg, k, v, seg_offset, l_s, l_x, B, H, d, causal, p_drop, seed, flags, workspace,
                                     workspace_bytes, out, lse, stream);
    if (elem_bytes == 4)
        return fwd_impl<float>(q_seg, k, v, seg_offset, l_s, l_x, B, H, d, causal, p_drop, seed, flags, workspace,
                               workspace_bytes, out, lse, stream);
    return fail(LSS_ERR_SHAPE, "elem_bytes = %d: 2 (bf16) or 4 (float)", elem_bytes);
}

int lss_segment_attn_bwd_ex(const void *q_seg, const void *k, const void *v, int64_t seg_offset, int64_t l_s, int64_t l_x,
                            int64_t B, int64_t H, int64_t d, int causal, double p_drop, uint64_t seed, int elem_bytes,
                            unsigned flags, void *workspace, size_t workspace_bytes, const void *out, const float *lse,
                            const void *dO, void *dq, float *dk_partial, float *dv_partial, void *stream)
{
    if (elem_bytes == 2)
        return bwd_impl<lss::bf16_t>(q_seg, k, v, seg_offset, l_s, l_x, B, H, d, causal, p_drop, seed, flags, workspace,
                                     workspace_bytes, out, lse, dO, dq, dk_partial, dv_partial, stream);
    if (elem_bytes == 4)
        return bwd_impl<float>(q_seg, k, v, seg_offset, l_s, l_x, B, H, d, causal, p_drop, seed, flags, workspace,
                               workspace_bytes, out, lse, dO, dq, dk_partial, dv_partial, stream);
    return fail(LSS_ERR_SHAPE, "elem_bytes = %d: 2 (bf16) or 4 (float)", elem_bytes);
}

int lss_segment_attn_fwd_dropout(const void *q_seg, const void *k, const void *v, int64_t seg_offset, int64_t l_s,
                                 int64_t l_x, int64_t B, int64_t H, int64_t d, int causal, double p_drop,
                                 uint64_t seed, int elem_bytes, void *out, float *lse, void *stream)
{
    return lss_segment_attn_fwd_ex(q_seg, k, v, seg_offset, l_s, l_x, B, H, d, causal, p_drop, seed, elem_bytes, 0u, nullptr,
                                   0, out, lse, stream);
}

int lss_segment_attn_bwd_dropout(const void *q_seg, const void *k, const void *v, int64_t seg_offset, int64_t l_s,
                                 int64_t l_x, int64_t B, int64_t H, int64_t d, int causal, double p_drop,
                                 uint64_t seed, int elem_bytes, const void *out, const float *lse, const void *dO,
                                 void *dq, float *dk_partial, float *dv_partial, void *stream)
{
    return lss_segment_attn_bwd_ex(q_seg, k, v, seg_offset, l_s, l_x, B, H, d, causal, p_drop, seed, elem_bytes, 0u, nullptr,
                                   0, out, lse, dO, dq, dk_partial, dv_partial, stream);
}

int lss_project_qkv(const void *x, const void *w_q, const void *w_kv, int64_t seg_offset, int64_t l_s, int64_t l_x,
                    int64_t B, int64_t H, int64_t d, void *q_seg, void *k, void *v, void *stream)
{
    if (int rc = check_shape(seg_offset, l_s, l_x, B, H, d)) return rc;
    const int64_t E = H * d;
    if (E % 128 != 0 || E > 65536)
        return fail(LSS_ERR_SHAPE, "projections: E_m = H*d = %lld is not a multiple of 128 or exceeds 65536", (long long)E);
    if (B * l_x >= (int64_t)1 << 31) return fail(LSS_ERR_SHAPE, "projections: B*l_x = %lld exceeds 2^31", (long long)(B * l_x));
    if (B == 0) return LSS_OK;
    if (!x || !w_q || !w_kv || !k || !v || (l_s > 0 && !q_seg)) return fail(LSS_ERR_NULL, "project_qkv: NULL tensor pointer");
    if (misaligned(x) || misaligned(w_q) || misaligned(w_kv) || misaligned(q_seg) || misaligned(k) || misaligned(v))
        return fail(LSS_ERR_ALIGN, "project_qkv: tensor pointers must be 16-byte aligned");
    using lss::bf16_t;
    const hipError_t e = lss::launch_project_qkv(static_cast<const bf16_t *>(x), static_cast<const bf16_t *>(w_q),
                                                 static_cast<const bf16_t *>(w_kv), seg_offset, (int)l_s, (int)l_x, (int)B,
                                                 (int)E, static_cast<bf16_t *>(q_seg), static_cast<bf16_t *>(k),
                                                 static_cast<bf16_t *>(v), static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(LSS_ERR_LAUNCH, "project_qkv launch failed: %s", hipGetErrorString(e));
    return LSS_OK;
}

int lss_project_bwd(const void *dq, const float *dk_partial, const float *dv_partial, const void *w_q, const void *w_kv,
                    int64_t l_s, int64_t l_x, int64_t rows_valid, int64_t B, int64_t H, int64_t d, float *dx_q,
                    float *dx_partial, void *stream)
{
    return lss_project_bwd_ex(dq, dk_partial, dv_partial, w_q, w_kv, l_s, l_x, rows_valid, B, H, d, 0u, dx_q, dx_partial, stream);
}

int lss_project_bwd_ex(const void *dq, const float *dk_partial, const float *dv_partial, const void *w_q, const void *w_kv,
                       int64_t l_s, int64_t l_x, int64_t rows_valid, int64_t B, int64_t H, int64_t d, unsigned flags,
                       float *dx_q, float *dx_partial, void *stream)
{
    if (int rc = check_shape(0, l_s, l_x, B, H, d)) return rc;
    if (int rc = check_flags(flags)) return rc;
    const int64_t E = H * d;
    if (E % 128 != 0 || E > 65536)
        return fail(LSS_ERR_SHAPE, "projections: E_m = H*d = %lld is not a multiple of 128 or exceeds 65536", (long long)E);
    if (rows_valid < 0 || rows_valid > l_x) return fail(LSS_ERR_RANGE, "project_bwd: rows_valid = %lld outside [0, %lld]", (long long)rows_valid, (long long)l_x);
    if (B == 0) return LSS_OK;
    if (!dk_partial || !dv_partial || !w_q || !w_kv || !dx_partial || (l_s > 0 && (!dq || !dx_q)))
        return fail(LSS_ERR_NULL, "project_bwd: NULL tensor pointer");
    if (misaligned(dq) || misaligned(dk_partial) || misaligned(dv_partial) || misaligned(w_q) || misaligned(w_kv) ||
        misaligned(dx_q) || misaligned(dx_partial))
        return fail(LSS_ERR_ALIGN, "project_bwd: tensor pointers must be 16-byte aligned");
    using lss::bf16_t;
    const hipError_t e = lss::launch_project_bwd(static_cast<const bf16_t *>(dq), dk_partial, dv_partial,
                                                 static_cast<const bf16_t *>(w_q), static_cast<const bf16_t *>(w_kv),
                                                 (int)l_s, (int)l_x, (int)rows_valid, (int)B, (int)E,
                                                 (flags & LSS_FLAG_SKIP_MASKED_TAIL) ? 1 : 0, dx_q, dx_partial,
                                                 static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(LSS_ERR_LAUNCH, "project_bwd launch failed: %s", hipGetErrorString(e));
    return LSS_OK;
}

// ---- segment-local row operations (Section 3, Principles 1 and 2)

int lss_embed_pe_fwd(const void *tok, const void *pe_table, int64_t seg_offset, int64_t l_s, int64_t l_x, int64_t B,
                     int64_t E_m, void *x, void *stream)
{
    if (l_s < 0 || l_x < 1 || B < 0 || E_m < 8 || E_m % 8 != 0 || l_s > INT32_MAX || B > INT32_MAX || E_m > 65536)
        return fail(LSS_ERR_SHAPE, "embed_pe: bad shape (l_s %lld, l_x %lld, B %lld, E_m %lld)", (long long)l_s,
                    (long long)l_x, (long long)B, (long long)E_m);
    if (seg_offset < 0 || seg_offset + l_s > l_x)
        return fail(LSS_ERR_RANGE, "embed_pe: rows [%lld, %lld) outside the table of %lld rows", (long long)seg_offset,
                    (long long)(seg_offset + l_s), (long long)l_x);
    if (B == 0 || l_s == 0) return LSS_OK;
    if (!tok || !pe_table || !x) return fail(LSS_ERR_NULL, "embed_pe: NULL tensor pointer");
    if (misaligned(tok) || misaligned(pe_table) || misaligned(x))
        return fail(LSS_ERR_ALIGN, "embed_pe: tensor pointers must be 16-byte aligned");
    using lss::bf16_t;
    const hipError_t e = lss::launch_embed_pe_fwd(static_cast<const bf16_t *>(tok), static_cast<const bf16_t *>(pe_table),
                                                  seg_offset, (int)l_s, (int)B, (int)E_m, static_cast<bf16_t *>(x),
                                                  static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(LSS_ERR_LAUNCH, "embed_pe launch failed: %s", hipGetErrorString(e));
    return LSS_OK;
}

int lss_embed_pe_bwd(const void *dx, int64_t l_s, int64_t B, int64_t E_m, float *dpe_rows, void *stream)
{
    if (l_s < 0 || B < 0 || E_m < 8 || E_m % 8 != 0 || l_s > INT32_MAX || B > INT32_MAX || E_m > 65536)
        return fail(LSS_ERR_SHAPE, "embed_pe_bwd: bad shape (l_s %lld, B %lld, E_m %lld)", (long long)l_s, (long long)B,
                    (long long)E_m);
    if (l_s == 0) return LSS_OK;
    if (!dpe_rows || (B > 0 && !dx)) return fail(LSS_ERR_NULL, "embed_pe_bwd: NULL tensor pointer");
    if (misaligned(dx) || misaligned(dpe_rows)) return fail(LSS_ERR_ALIGN, "embed_pe_bwd: tensor pointers must be 16-byte aligned");
    const hipError_t e = lss::launch_embed_pe_bwd(static_cast<const lss::bf16_t *>(dx), (int)l_s, (int)B, (int)E_m, dpe_rows,
                                                  static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(LSS_ERR_LAUNCH, "embed_pe_bwd launch failed: %s", hipGetErrorString(e));
    return LSS_OK;
}

int lss_residual_dropout_add(const void *x, const void *delta, int64_t seg_offset, int64_t l_s, int64_t B, int64_t E_m,
                             double p_drop, uint64_t seed, void *out, void *stream)
{
    if (l_s < 0 || B < 0 || E_m < 8 || E_m % 8 != 0 || l_s > INT32_MAX || B > INT32_MAX || E_m > 65536)
        return fail(LSS_ERR_SHAPE, "residual_dropout_add: bad shape (l_s %lld, B %lld, E_m %lld)", (long long)l_s, (long long)B,
                    (long long)E_m);
    if (seg_offset < 0 || seg_offset + l_s > (int64_t)UINT32_MAX)
        return fail(LSS_ERR_RANGE, "residual_dropout_add: seg_offset = %lld", (long long)seg_offset);
    if (int rc = check_dropout(p_drop)) return rc;
    if (B == 0 || l_s == 0) return LSS_OK;
    if (!delta || !out) return fail(LSS_ERR_NULL, "residual_dropout_add: NULL tensor pointer");
    if (misaligned(x) || misaligned(delta) || misaligned(out))
        return fail(LSS_ERR_ALIGN, "residual_dropout_add: tensor pointers must be 16-byte aligned");
    using lss::bf16_t;
    const hipError_t e = lss::launch_residual_add(static_cast<const bf16_t *>(x), static_cast<const bf16_t *>(delta),
                                                  dropout_args(p_drop, seed), seg_offset, (int)l_s, (int)B, (int)E_m,
                                                  static_cast<bf16_t *>(out), static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(LSS_ERR_LAUNCH, "residual_dropout_add launch failed: %s", hipGetErrorString(e));
    return LSS_OK;
}

static int check_layernorm(const char *what, int64_t rows, int64_t E_m)
{
    if (rows < 0 || E_m < 8 || E_m % 8 != 0 || E_m > lss::layernorm_max_columns())
        return fail(LSS_ERR_SHAPE, "%s: rows = %lld, E_m = %lld (need E_m a multiple of 8, at most %d)", what, (long long)rows,
                    (long long)E_m, lss::layernorm_max_columns());
    return LSS_OK;
}

int lss_layernorm_fwd(const void *x, const float *gamma, const float *beta, double eps, int64_t rows, int64_t E_m, void *y,
                      float *mean, float *rstd, void *stream)
{
    if (int rc = check_layernorm("layernorm_fwd", rows, E_m)) return rc;
    if (!(eps >= 0.0)) return fail(LSS_ERR_RANGE, "layernorm_fwd: eps = %g", eps);
    if (rows == 0) return LSS_OK;
    if (!x || !gamma || !beta || !y || !mean || !rstd) return fail(LSS_ERR_NULL, "layernorm_fwd: NULL tensor pointer");
    if (misaligned(x) || misaligned(gamma) || misaligned(beta) || misaligned(y))
        return fail(LSS_ERR_ALIGN, "layernorm_fwd: tensor pointers must be 16-byte aligned");
    using lss::bf16_t;
    const hipError_t e = lss::launch_layernorm_fwd(static_cast<const bf16_t *>(x), gamma, beta, (float)eps, rows, (int)E_m,
                                                   static_cast<bf16_t *>(y), mean, rstd, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(LSS_ERR_LAUNCH, "layernorm_fwd launch failed: %s", hipGetErrorString(e));
    return LSS_OK;
}

size_t lss_layernorm_bwd_scratch_bytes(int64_t rows, int64_t E_m)
{
    if (rows <= 0 || E_m <= 0 || E_m > lss::layernorm_max_columns()) return 0;
    return lss::layernorm_bwd_scratch_bytes(rows, (int)E_m);
}

int lss_layernorm_bwd(const void *x, const float *gamma, const float *mean, const float *rstd, const void *dy, int64_t rows,
                      int64_t E_m, void *dx, float *dgamma, float *dbeta, void *scratch, size_t scratch_bytes, void *stream)
{
    if (int rc = check_layernorm("layernorm_bwd", rows, E_m)) return rc;
    if (!dgamma || !dbeta) return fail(LSS_ERR_NULL, "layernorm_bwd: NULL gradient pointer");
    if (rows > 0) {
        if (!x || !gamma || !mean || !rstd || !dy || !dx) return fail(LSS_ERR_NULL, "layernorm_bwd: NULL tensor pointer");
        if (misaligned(x) || misaligned(gamma) || misaligned(dy) || misaligned(dx) || misaligned(scratch))
            return fail(LSS_ERR_ALIGN, "layernorm_bwd: tensor pointers must be 16-byte aligned");
        const size_t need = lss::layernorm_bwd_scratch_bytes(rows, (int)E_m);
        if (!scratch || scratch_bytes < need)
            return fail(LSS_ERR_WORKSPACE, "layernorm_bwd: scratch of %zu bytes, need %zu", scratch ? scratch_bytes : (size_t)0, need);
    }
    using lss::bf16_t;
    const hipError_t e = lss::launch_layernorm_bwd(static_cast<const bf16_t *>(x), gamma, mean, rstd,
                                                   static_cast<const bf16_t *>(dy), rows, (int)E_m, static_cast<bf16_t *>(dx),
                                                   dgamma, dbeta, static_cast<float *>(scratch), static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(LSS_ERR_LAUNCH, "layernorm_bwd launch failed: %s", hipGetErrorString(e));
    return LSS_OK;
}

static int check_linear(const char *what, const void *a, const void *w, const void *c, int64_t rows, int64_t K, int64_t N)
{
    if (rows < 0 || rows > INT32_MAX || K < 128 || N < 128 || K % 128 != 0 || N % 128 != 0 || K > 65536 || N > 65536)
        return fail(LSS_ERR_SHAPE, "%s: rows = %lld, K = %lld, N = %lld (K, N multiples of 128, at most 65536)", what,
                    (long long)rows, (long long)K, (long long)N);
    if (rows == 0) return LSS_OK;
    if (!a || !w || !c) return fail(LSS_ERR_NULL, "%s: NULL tensor pointer", what);
    if (misaligned(a) || misaligned(w) || misaligned(c)) return fail(LSS_ERR_ALIGN, "%s: tensor pointers must be 16-byte aligned", what);
    return LSS_OK;
}

static int linear_fwd_impl(const char *what, const void *a, const void *w, int64_t rows, int64_t K, int64_t N, void *c,
                           void *gelu_c, bool fused, void *stream)
{
    if (int rc = check_linear(what, a, w, c, rows, K, N)) return rc;
    if (rows == 0) return LSS_OK;
    if (fused && !gelu_c) return fail(LSS_ERR_NULL, "%s: NULL tensor pointer", what);
    if (misaligned(gelu_c)) return fail(LSS_ERR_ALIGN, "%s: tensor pointers must be 16-byte aligned", what);
    using lss::bf16_t;
    const hipError_t e = lss::launch_linear_fwd(static_cast<const bf16_t *>(a), static_cast<const bf16_t *>(w), (int)rows, (int)K,
                                                (int)N, static_cast<bf16_t *>(c), static_cast<bf16_t *>(gelu_c),
                                                static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(LSS_ERR_LAUNCH, "%s launch failed: %s", what, hipGetErrorString(e));
    return LSS_OK;
}

static int linear_bwd_impl(const char *what, const void *dc, const void *w, const void *gelu_u, bool fused, int64_t rows,
                           int64_t K, int64_t N, void *da, void *stream)
{
    if (int rc = check_linear(what, dc, w, da, rows, K, N)) return rc;
    if (rows == 0) return LSS_OK;
    if (fused && !gelu_u) return fail(LSS_ERR_NULL, "%s: NULL tensor pointer", what);
    if (misaligned(gelu_u)) return fail(LSS_ERR_ALIGN, "%s: tensor pointers must be 16-byte aligned", what);
    using lss::bf16_t;
    const hipError_t e = lss::launch_linear_bwd_input(static_cast<const bf16_t *>(dc), static_cast<const bf16_t *>(w),
                                                      static_cast<const bf16_t *>(gelu_u), (int)rows, (int)K, (int)N,
                                                      static_cast<bf16_t *>(da), static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(LSS_ERR_LAUNCH, "%s launch failed: %s", what, hipGetErrorString(e));
    return LSS_OK;
}

int lss_linear_fwd(const void *a, const void *w, int64_t rows, int64_t K, int64_t N, void *c, void *stream)
{
    return linear_fwd_impl("linear_fwd", a, w, rows, K, N, c, nullptr, false, stream);
}

int lss_linear_gelu_fwd(const void *a, const void *w, int64_t rows, int64_t K, int64_t N, void *u, void *g, void *stream)
{
    return linear_fwd_impl("linear_gelu_fwd", a, w, rows, K, N, u, g, true, stream);
}

int lss_linear_bwd_input(const void *dc, const void *w, int64_t rows, int64_t K, int64_t N, void *da, void *stream)
{
    return linear_bwd_impl("linear_bwd_input", dc, w, nullptr, false, rows, K, N, da, stream);
}

int lss_linear_bwd_input_gelu(const void *dc, const void *w, const void *u, int64_t rows, int64_t K, int64_t N, void *du,
                              void *stream)
{
    return linear_bwd_impl("linear_bwd_input_gelu", dc, w, u, true, rows, K, N, du, stream);
}

size_t lss_linear_bwd_weight_scratch_bytes(int64_t rows, int64_t K, int64_t N)
{
    if (rows < 1 || rows > INT32_MAX || K < 128 || N < 128 || K % 128 != 0 || N % 128 != 0 || K > 65536 || N > 65536) return 0;
    return lss::linear_bwd_weight_scratch_bytes((int)rows, (int)K, (int)N);
}

int lss_linear_bwd_weight(const void *a, const void *dc, int64_t rows, int64_t K, int64_t N, float *dw, void *scratch,
                          size_t scratch_bytes, void *stream)
{
    if (rows < 0 || rows > INT32_MAX || K < 128 || N < 128 || K % 128 != 0 || N % 128 != 0 || K > 65536 || N > 65536)
        return fail(LSS_ERR_SHAPE, "linear_bwd_weight: rows = %lld, K = %lld, N = %lld (K, N multiples of 128, at most 65536)",
                    (long long)rows, (long long)K, (long long)N);
    if (!dw) return fail(LSS_ERR_NULL, "linear_bwd_weight: NULL tensor pointer");
    if (misaligned(dw)) return fail(LSS_ERR_ALIGN, "linear_bwd_weight: tensor pointers must be 16-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (rows == 0) {    // no rows: the gradient is zero (written by the sum kernel over one part without valid rows)
        const int64_t none = 0;
        const float *part = dw;
        const hipError_t e = lss::launch_reduce(&part, 1, &none, K, 1, 1, N, dw, st);
        if (e != hipSuccess) return fail(LSS_ERR_LAUNCH, "linear_bwd_weight launch failed: %s", hipGetErrorString(e));
        return LSS_OK;
    }
    if (!a || !dc) return fail(LSS_ERR_NULL, "linear_bwd_weight: NULL tensor pointer");
    if (misaligned(a) || misaligned(dc) || misaligned(scratch))
        return fail(LSS_ERR_ALIGN, "linear_bwd_weight: tensor pointers must be 16-byte aligned");
    const size_t need = lss::linear_bwd_weight_scratch_bytes((int)rows, (int)K, (int)N);
    if (need > 0 && (!scratch || scratch_bytes < need))
        return fail(LSS_ERR_WORKSPACE, "linear_bwd_weight: scratch of %zu bytes, need %zu", scratch ? scratch_bytes : (size_t)0, need);
    using lss::bf16_t;
    const hipError_t e = lss::launch_linear_bwd_weight(static_cast<const bf16_t *>(a), static_cast<const bf16_t *>(dc), (int)rows,
                                                       (int)K, (int)N, dw, static_cast<float *>(scratch), st);
    if (e != hipSuccess) return fail(LSS_ERR_LAUNCH, "linear_bwd_weight launch failed: %s", hipGetErrorString(e));
    return LSS_OK;
}

static int check_gelu(const char *what, int64_t n)
{
    if (n < 0 || n % 8 != 0) return fail(LSS_ERR_SHAPE, "%s: n = %lld is not a non-negative multiple of 8", what, (long long)n);
    return LSS_OK;
}

int lss_gelu_fwd(const void *u, int64_t n, void *g, void *stream)
{
    if (int rc = check_gelu("gelu_fwd", n)) return rc;
    if (n == 0) return LSS_OK;
    if (!u || !g) return fail(LSS_ERR_NULL, "gelu_fwd: NULL tensor pointer");
    if (misaligned(u) || misaligned(g)) return fail(LSS_ERR_ALIGN, "gelu_fwd: tensor pointers must be 16-byte aligned");
    const hipError_t e = lss::launch_gelu_fwd(static_cast<const lss::bf16_t *>(u), n, static_cast<lss::bf16_t *>(g),
                                              static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(LSS_ERR_LAUNCH, "gelu_fwd launch failed: %s", hipGetErrorString(e));
    return LSS_OK;
}

int lss_gelu_bwd(const void *u, const void *dg, int64_t n, void *du, void *stream)
{
    if (int rc = check_gelu("gelu_bwd", n)) return rc;
    if (n == 0) return LSS_OK;
    if (!u || !dg || !du) return fail(LSS_ERR_NULL, "gelu_bwd: NULL tensor pointer");
    if (misaligned(u) || misaligned(dg) || misaligned(du)) return fail(LSS_ERR_ALIGN, "gelu_bwd: tensor pointers must be 16-byte aligned");
    const hipError_t e = lss::launch_gelu_bwd(static_cast<const lss::bf16_t *>(u), static_cast<const lss::bf16_t *>(dg), n,
                                              static_cast<lss::bf16_t *>(du), static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(LSS_ERR_LAUNCH, "gelu_bwd launch failed: %s", hipGetErrorString(e));
    return LSS_OK;
}

size_t lss_project_bwd_weight_scratch_bytes(int64_t l_s, int64_t l_x, int64_t B, int64_t H, int64_t d)
{
    const int64_t E = H * d;
    if (l_s < 0 || l_x < 1 || B < 1 || H < 1 || d < 1 || l_s > l_x || l_x > INT32_MAX || B > INT32_MAX || E % 128 != 0 || E > 65536)
        return 0;
    return lss::project_bwd_weight_scratch_bytes((int)l_s, (int)l_x, (int)B, (int)E);
}

int lss_project_bwd_weight(const void *x, const void *dq, const float *dk_partial, const float *dv_partial, int64_t seg_offset,
                           int64_t l_s, int64_t l_x, int64_t rows_valid, int64_t B, int64_t H, int64_t d, float *dw_q,
                           float *dw_kv, void *scratch, size_t scratch_bytes, void *stream)
{
    if (int rc = check_shape(seg_offset, l_s, l_x, B, H, d)) return rc;
    const int64_t E = H * d;
    if (E % 128 != 0 || E > 65536)
        return fail(LSS_ERR_SHAPE, "projections: E_m = H*d = %lld is not a multiple of 128 or exceeds 65536", (long long)E);
    if (rows_valid < 0 || rows_valid > l_x)
        return fail(LSS_ERR_RANGE, "project_bwd_weight: rows_valid = %lld outside [0, %lld]", (long long)rows_valid, (long long)l_x);
    if (!dw_q || !dw_kv) return fail(LSS_ERR_NULL, "project_bwd_weight: NULL gradient pointer");
    if (misaligned(dw_q) || misaligned(dw_kv)) return fail(LSS_ERR_ALIGN, "project_bwd_weight: tensor pointers must be 16-byte aligned");
    const bool has_q = B > 0 && l_s > 0, has_kv = B > 0 && rows_valid > 0;
    if ((has_q && (!x || !dq)) || (has_kv && (!x || !dk_partial || !dv_partial)))
        return fail(LSS_ERR_NULL, "project_bwd_weight: NULL tensor pointer");
    if (misaligned(x) || misaligned(dq) || misaligned(dk_partial) || misaligned(dv_partial) || misaligned(scratch))
        return fail(LSS_ERR_ALIGN, "project_bwd_weight: tensor pointers must be 16-byte aligned");
    const size_t need = B > 0 ? lss::project_bwd_weight_scratch_needed(has_q ? (int)l_s : 0, has_kv ? (int)rows_valid : 0, (int)B, (int)E) : 0;
    if (need > 0 && (!scratch || scratch_bytes < need))
        return fail(LSS_ERR_WORKSPACE, "project_bwd_weight: scratch of %zu bytes, need %zu", scratch ? scratch_bytes : (size_t)0, need);
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e = hipSuccess;
    const int64_t none = 0;     // a gradient without rows is zero: written by the sum kernel over one part without valid rows
    if (!has_q) {
        const float *part = dw_q;
        e = lss::launch_reduce(&part, 1, &none, E, 1, 1, E, dw_q, st);
    }
    if (e == hipSuccess && !has_kv) {
        const float *part = dw_kv;
        e = lss::launch_reduce(&part, 1, &none, E, 1, 1, 2 * E, dw_kv, st);
    }
    using lss::bf16_t;
    if (e == hipSuccess && (has_q || has_kv))
        e = lss::launch_project_bwd_weight(static_cast<const bf16_t *>(x), static_cast<const bf16_t *>(dq), dk_partial, dv_partial,
                                           seg_offset, has_q ? (int)l_s : 0, (int)l_x, has_kv ? (int)rows_valid : 0, (int)B, (int)E,
                                           dw_q, dw_kv, static_cast<float *>(scratch), st);
    if (e != hipSuccess) return fail(LSS_ERR_LAUNCH, "project_bwd_weight launch failed: %s", hipGetErrorString(e));
    return LSS_OK;
}

int lss_reduce_partials(const float *const *parts, int n, const int64_t *rows_valid, int64_t l_x, int64_t B,
                        int64_t H, int64_t d, float *out, void *stream)
{
    if (n < 1) return fail(LSS_ERR_SHAPE, "reduce: n = %d, need at least one part", n);
    if (l_x < 1 || B < 0 || H < 1 || d < 4 || d % 4 != 0) return fail(LSS_ERR_SHAPE, "reduce: bad shape");
    if (!parts || !out) return fail(LSS_ERR_NULL, "reduce: NULL pointer");
    if (misaligned(out)) return fail(LSS_ERR_ALIGN, "reduce: out must be 16-byte aligned");
    for (int i = 0; i < n; ++i) {
        if (!parts[i]) return fail(LSS_ERR_NULL, "reduce: parts[%d] is NULL", i);
        if (misaligned(parts[i])) return fail(LSS_ERR_ALIGN, "reduce: parts[%d] must be 16-byte aligned", i);
        if (i > 0 && parts[i] == out) return fail(LSS_ERR_RANGE, "reduce: out may alias parts[0] only");
    }
    const hipError_t e = lss::launch_reduce(parts, n, rows_valid, l_x, B, H, d, out, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(LSS_ERR_LAUNCH, "reduce launch failed: %s", hipGetErrorString(e));
    return LSS_OK;
}

} // extern "C"
