// Optional per-kernel timing with HIP events (host code only).
//
// Off by default.  While enabled, every kernel launch of the library is
// bracketed by two events recorded on the launch stream; hdqt_profile_collect
// waits for them, sums the elapsed times per kernel and clears the list.  This
// is the only state the library keeps, and only while the caller asked for it.
// The switch and the event lists are process-wide: launches from any thread and on any
// stream are recorded while it is on (the lists are guarded by one mutex, the switch is
// atomic), and hdqt_profile_collect returns all of them.  Turn it on around a region that
// one thread controls; the events of two threads' launches are not kept apart.

#include "../../include/hdqt.h"
#include "common.hpp"

#include <atomic>
#include <mutex>
#include <string.h>
#include <vector>

namespace hdqt {

namespace {
struct Pending { int id; hipEvent_t start, stop; };
std::mutex g_mu;
std::atomic<bool> g_enabled{false};
std::vector<Pending> g_pending;
std::vector<Pending> g_open;     // begun, not yet ended (per launch, LIFO)
} // namespace

const char* kernel_name(int id)
{
    static const char* names[K_COUNT] = {
        "zero", "fwht_row_absmax", "fwht_row_quant", "fwht_col_absmax", "fwht_col_quant",
        "plain_absmax", "plain_quant", "gemm_tiled_aligned", "gemm_tiled_generic", "reduce_splits",
        "gemm_i4", "fwht_dual_absmax", "fwht_dual_quant", "gemm_i4_fwd", "gemm_i4_bwd_input",
        "gemm_i4_bwd_weight", "fwht_dual_absmax_X", "fwht_dual_absmax_W", "fwht_dual_absmax_G",
        "fwht_dual_quant_X", "fwht_dual_quant_W", "fwht_dual_quant_G", "fwht_dual_absmax_batch",
        "fwht_dual_quant_batch", "requant_tile_sums", "requant_quantize_sum", "im2col", "relu_mask"};
    return (id >= 0 && id < K_COUNT) ? names[id] : "?";
}

bool profiling_enabled() { return g_enabled.load(std::memory_order_relaxed); }

void profile_begin(int id, hipStream_t stream)
{
    std::lock_guard<std::mutex> lock(g_mu);
    Pending p{id, nullptr, nullptr};
    if (hipEventCreate(&p.start) != hipSuccess) return;
    if (hipEventCreate(&p.stop) != hipSuccess) { (void)hipEventDestroy(p.start); return; }
    (void)hipEventRecord(p.start, stream);
    g_open.push_back(p);
}

void profile_end(int id, hipStream_t stream)
{
    std::lock_guard<std::mutex> lock(g_mu);
    for (size_t k = g_open.size(); k-- > 0;) {
        if (g_open[k].id == id) {
            Pending p = g_open[k];
            g_open.erase(g_open.begin() + (long)k);
            (void)hipEventRecord(p.stop, stream);
            g_pending.push_back(p);
            return;
        }
    }
}

} // namespace hdqt

extern "C" {

int hdqt_profile_enable(int on)
{
    std::lock_guard<std::mutex> lock(hdqt::g_mu);
    hdqt::g_enabled.store(on != 0, std::memory_order_relaxed);
    return HDQT_OK;
}

int hdqt_profile_collect(hdqt_kernel_time_t* rows, int max_rows)
{
    std::lock_guard<std::mutex> lock(hdqt::g_mu);
    double total[hdqt::K_COUNT] = {0};
    long launches[hdqt::K_COUNT] = {0};
    for (const hdqt::Pending& p : hdqt::g_pending) {
        float ms = 0.0f;
        if (hipEventSynchronize(p.stop) == hipSuccess &&
            hipEventElapsedTime(&ms, p.start, p.stop) == hipSuccess) {
            total[p.id] += ms;
            launches[p.id] += 1;
        }
        (void)hipEventDestroy(p.start);
        (void)hipEventDestroy(p.stop);
    }
    hdqt::g_pending.clear();
    int n = 0;
    for (int id = 0; id < hdqt::K_COUNT; ++id) {
        if (!launches[id]) continue;
        if (rows && n < max_rows) {
            strncpy(rows[n].name, hdqt::kernel_name(id), sizeof(rows[n].name) - 1);
            rows[n].name[sizeof(rows[n].name) - 1] = 0;
            rows[n].launches = launches[id];
            rows[n].total_ms = total[id];
        }
        ++n;
    }
    return n;
}

} // extern "C"
