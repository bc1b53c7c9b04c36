// Optional per-kernel timing: HIP events recorded on the launch stream around every kernel
// the library launches, summed per kernel.  Off by default; a benchmark turns it on.
#include "lss_attn.h"
#include "lss_kernels.h"
#include "lss_timing.h"

#include <atomic>
#include <mutex>
#include <vector>

namespace lss {
namespace {

struct Record { int id; hipEvent_t start, stop; };

std::atomic<uint64_t> g_mask{0};         // bit i set: kernel id i is timed
std::mutex g_mu;
std::vector<Record> g_open;             // recorded, not yet read back
std::vector<hipEvent_t> g_free;         // events ready for reuse
thread_local hipEvent_t t_start = nullptr;
double g_total_ms[K_COUNT] = {0};
int64_t g_count[K_COUNT] = {0};

// the __global__ function each id stands for; ":role" where entry points share one function
const char *const kNames[K_COUNT] = {"fwd_kernel", "fwd_merge_kernel", "bwd_rowdot_kernel", "bwd_dq_kernel",
                                     "bwd_dq_merge_kernel", "bwd_dkv_kernel", "reduce_partials_kernel",
                                     "bwd_main_bf16_kernel", "proj_gemm_kernel:project_qkv", "proj_gemm_kernel:project_bwd",
                                     "embed_pe_fwd_kernel", "embed_pe_bwd_kernel", "layernorm_fwd_kernel",
                                     "layernorm_bwd_kernel", "layernorm_bwd_params_kernel", "gelu_fwd_kernel",
                                     "gelu_bwd_kernel", "proj_gemm_kernel:linear_fwd", "proj_gemm_kernel:linear_bwd_input",
                                     "residual_add_kernel", "wgrad_gemm_kernel", "fwd_bf16_kernel", "bwd_prep_bf16_kernel"};

hipEvent_t get_event()
{
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_free.empty()) {
        hipEvent_t e = g_free.back();
        g_free.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

// Wait for every recorded pair and add its elapsed time to the per-kernel totals.
int collect()
{
    std::vector<Record> open;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        open.swap(g_open);
    }
    int rc = LSS_OK;
    for (const Record &r : open) {
        float ms = 0.f;
        if (hipEventSynchronize(r.stop) == hipSuccess && hipEventElapsedTime(&ms, r.start, r.stop) == hipSuccess) {
            g_total_ms[r.id] += ms;
            g_count[r.id] += 1;
        } else {
            rc = LSS_ERR_LAUNCH;
        }
        std::lock_guard<std::mutex> lock(g_mu);
        g_free.push_back(r.start);
        g_free.push_back(r.stop);
    }
    return rc;
}

} // namespace

void timing_begin(int id, hipStream_t st)
{
    if (!((g_mask.load(std::memory_order_relaxed) >> id) & 1u)) return;
    t_start = get_event();
    if (t_start) (void)hipEventRecord(t_start, st);
}

void timing_end(int id, hipStream_t st)
{
    if (!((g_mask.load(std::memory_order_relaxed) >> id) & 1u) || !t_start) return;
    hipEvent_t stop = get_event();
    if (!stop) return;
    (void)hipEventRecord(stop, st);
    std::lock_guard<std::mutex> lock(g_mu);
    g_open.push_back(Record{id, t_start, stop});
    t_start = nullptr;
}

} // namespace lss

extern "C" {

int lss_timing_enable(int on)
{
    lss::g_mask.store(on != 0 ? ~(uint64_t)0 : (uint64_t)0);
    return LSS_OK;
}

int lss_timing_select(uint64_t kernel_mask)
{
    lss::g_mask.store(kernel_mask);
    return LSS_OK;
}

int lss_timing_reset(void)
{
    const int rc = lss::collect();
    for (int i = 0; i < lss::K_COUNT; ++i) { lss::g_total_ms[i] = 0; lss::g_count[i] = 0; }
    return rc;
}

int lss_timing_read(int kernel_id, double *total_ms, int64_t *launches)
{
    if (kernel_id < 0 || kernel_id >= lss::K_COUNT || !total_ms || !launches) return LSS_ERR_RANGE;
    const int rc = lss::collect();
    *total_ms = lss::g_total_ms[kernel_id];
    *launches = lss::g_count[kernel_id];
    return rc;
}

const char *lss_timing_kernel_name(int kernel_id)
{
    return (kernel_id >= 0 && kernel_id < lss::K_COUNT) ? lss::kNames[kernel_id] : nullptr;
}

} // extern "C"
