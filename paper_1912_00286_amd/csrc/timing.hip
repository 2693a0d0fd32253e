// Optional per-kernel-class timing with HIP events recorded on the caller's
// stream around each launch.  Off by default; when off the only cost is one
// branch per launch.  Used by the benchmark to report the measured duration of
// the dominant kernel class next to its algorithmic work.
#include <mutex>
#include <vector>

#include "common.h"

namespace lstm {
namespace {

struct Span {
    hipEvent_t beg, end;
    int cls;
};

std::mutex g_mu;
bool g_on = false;
std::vector<Span> g_open;                 // recorded, not yet read
std::vector<hipEvent_t> g_pool;           // reusable events
struct Acc { int64_t launches = 0; double ms = 0, flops = 0, bytes = 0; } g_acc[KC_COUNT];

hipEvent_t get_event() {
    if (!g_pool.empty()) {
        hipEvent_t e = g_pool.back();
        g_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    // timing only: no system-scope fence when the event completes (it would add its own latency
    // to every bracketed launch)
    if (hipEventCreateWithFlags(&e, hipEventDisableSystemFence) != hipSuccess) return nullptr;
    return e;
}

}  // namespace

bool timing_enabled() { return g_on; }

KernelTimer::KernelTimer(int cls, hipStream_t s, double flops, double bytes) : cls_(cls), stream_(s), beg_(nullptr) {
    if (!g_on) return;
    std::lock_guard<std::mutex> lk(g_mu);
    beg_ = get_event();
    if (!beg_) return;
    g_acc[cls].launches += 1;
    g_acc[cls].flops += flops;
    g_acc[cls].bytes += bytes;
    (void)hipEventRecord((hipEvent_t)beg_, s);
}

KernelTimer::~KernelTimer() {
    if (!beg_) return;
    std::lock_guard<std::mutex> lk(g_mu);
    hipEvent_t e = get_event();
    if (!e) return;
    (void)hipEventRecord(e, stream_);
    g_open.push_back(Span{(hipEvent_t)beg_, e, cls_});
}

}  // namespace lstm

using namespace lstm;

extern "C" int lstm_timing_enable(int32_t on) {
    std::lock_guard<std::mutex> lk(g_mu);
    for (auto &sp : g_open) {
        g_pool.push_back(sp.beg);
        g_pool.push_back(sp.end);
    }
    g_open.clear();
    for (auto &a : g_acc) a = Acc();
    g_on = on != 0;
    return LSTM_OK;
}

extern "C" int lstm_timing_read(int32_t kernel_class, int64_t *launches, double *total_ms, double *flops, double *bytes) {
    if (kernel_class < 0 || kernel_class >= KC_COUNT || !launches || !total_ms || !flops || !bytes) {
        set_error("lstm_timing_read: invalid argument");
        return LSTM_ERR_INVALID;
    }
    std::lock_guard<std::mutex> lk(g_mu);
    // fold every finished span into the accumulators (waits for the recorded work)
    for (auto &sp : g_open) {
        LSTM_HIP_TRY(hipEventSynchronize(sp.end));
        float ms = 0.0f;
        LSTM_HIP_TRY(hipEventElapsedTime(&ms, sp.beg, sp.end));
        g_acc[sp.cls].ms += ms;
        g_pool.push_back(sp.beg);
        g_pool.push_back(sp.end);
    }
    g_open.clear();
    *launches = g_acc[kernel_class].launches;
    *total_ms = g_acc[kernel_class].ms;
    *flops = g_acc[kernel_class].flops;
    *bytes = g_acc[kernel_class].bytes;
    return LSTM_OK;
}
