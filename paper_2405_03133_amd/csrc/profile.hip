// Optional per-kernel-class timing with HIP events on the caller's stream.
// Off by default; when on, every launch of the hot path is bracketed by a pair
// of events and tagged with the algorithmic FLOPs and bytes of that launch, so
// a benchmark can report achieved TFLOP/s and GB/s per kernel class without an
// external profiler.
#include "lory_internal.h"

#include <string.h>

#include <vector>

namespace lory {
namespace prof {

namespace {

struct Record {
    int cls;
    hipEvent_t start, stop;
    double flops, bytes;
};

bool g_on = false;
std::vector<Record> g_records;
std::vector<hipEvent_t> g_pool;

const char *const kNames[kNumClasses] = {"route",     "merge",     "gemm_gate_up", "swiglu_fwd", "gemm_down",
                                         "gemm_dA",   "swiglu_bwd", "gemm_dX",   "gemm_dW_gate_up",
                                         "gemm_dW_down", "scatter_dots", "dw_reduce", "route_bwd", "dense_skinny",
                                         "fused_gate_up", "fused_down", "fused_dA", "fused_dX", "fused_dW_dots"};

// Events are created when timing is switched on (and by lory_profile_read, which returns
// them to the pool), never inside a launch: a launch only takes events from the pool and
// goes untimed when the pool is empty.
constexpr size_t kPoolEvents = 4096;   // 2048 timed launches between two reads

hipEvent_t get_event()
{
    if (g_pool.empty()) return nullptr;
    hipEvent_t e = g_pool.back();
    g_pool.pop_back();
    return e;
}

void fill_pool()
{
    g_pool.reserve(kPoolEvents);
    g_records.reserve(kPoolEvents / 2);
    while (g_pool.size() < kPoolEvents) {
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) break;
        g_pool.push_back(e);
    }
}

}  // namespace

bool enabled() { return g_on; }

Range::Range(hipStream_t st, int cls, double flops, double bytes) : st_(st), idx_(-1)
{
    if (!g_on) return;
    Record r;
    r.cls = cls;
    r.flops = flops;
    r.bytes = bytes;
    if (g_pool.size() < 2 || g_records.size() == g_records.capacity()) return;  // untimed launch
    r.start = get_event();
    r.stop = get_event();
    hipEventRecord(r.start, st);
    g_records.push_back(r);
    idx_ = (int)g_records.size() - 1;
}

Range::~Range()
{
    if (idx_ >= 0) hipEventRecord(g_records[idx_].stop, st_);
}

int set_enabled(int on)
{
    g_on = on != 0;
    if (g_on) fill_pool();
    return LORY_OK;
}

int read(lory_kernel_stat *out, int max_out, int *n_out)
{
    lory_kernel_stat acc[kNumClasses];
    memset(acc, 0, sizeof(acc));
    for (int c = 0; c < kNumClasses; ++c) strncpy(acc[c].name, kNames[c], sizeof(acc[c].name) - 1);
    int rc = LORY_OK;
    for (const Record &r : g_records) {
        float ms = 0.f;
        if (hipEventSynchronize(r.stop) != hipSuccess ||
            hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) {
            rc = LORY_ERR_DEVICE;
        } else {
            acc[r.cls].launches += 1;
            acc[r.cls].ms += ms;
            acc[r.cls].flops += r.flops;
            acc[r.cls].bytes += r.bytes;
        }
        g_pool.push_back(r.start);
        g_pool.push_back(r.stop);
    }
    g_records.clear();
    int n = 0;
    for (int c = 0; c < kNumClasses && n < max_out; ++c)
        if (acc[c].launches > 0) out[n++] = acc[c];
    *n_out = n;
    return rc;
}

}  // namespace prof
}  // namespace lory
