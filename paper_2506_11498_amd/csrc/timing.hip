// Optional per-kernel timing with HIP events, recorded on the stream each kernel is launched on.
// Off by default; the benchmark switches it on to report the duration of individual kernels.
#include "../../include/lrsa.h"
#include "common.h"

#include <mutex>
#include <vector>

namespace lrsa {

namespace {
struct Record {
    const char* name;
    hipEvent_t beg, end;
};
std::mutex g_mu;
bool g_on = false;
std::vector<Record> g_rec;       // records in use
std::vector<Record> g_pool;      // events kept for reuse
constexpr size_t kMaxRecords = 4096;
}  // namespace

ScopedKernelTimer::ScopedKernelTimer(const char* name, hipStream_t st) : st_(st), slot_(-1) {
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_on || g_rec.size() >= kMaxRecords) return;
    Record r;
    if (!g_pool.empty()) {
        r = g_pool.back();
        g_pool.pop_back();
    } else if (hipEventCreate(&r.beg) != hipSuccess || hipEventCreate(&r.end) != hipSuccess) {
        return;
    }
    r.name = name;
    if (hipEventRecord(r.beg, st) != hipSuccess) { g_pool.push_back(r); return; }
    g_rec.push_back(r);
    slot_ = int(g_rec.size()) - 1;
}

ScopedKernelTimer::~ScopedKernelTimer() {
    if (slot_ < 0) return;
    std::lock_guard<std::mutex> lk(g_mu);
    if (slot_ < int(g_rec.size())) (void)hipEventRecord(g_rec[slot_].end, st_);
}

}  // namespace lrsa

extern "C" {

int lrsa_timing_enable(int on) {
    std::lock_guard<std::mutex> lk(lrsa::g_mu);
    for (auto& r : lrsa::g_rec) lrsa::g_pool.push_back(r);
    lrsa::g_rec.clear();
    lrsa::g_on = on != 0;
    return LRSA_OK;
}

int lrsa_timing_count(void) {
    std::lock_guard<std::mutex> lk(lrsa::g_mu);
    return int(lrsa::g_rec.size());
}

int lrsa_timing_read(int i, const char** name, float* ms) {
    std::lock_guard<std::mutex> lk(lrsa::g_mu);
    if (i < 0 || i >= int(lrsa::g_rec.size()) || !name || !ms) return LRSA_ERR_INVALID_ARG;
    const auto& r = lrsa::g_rec[i];
    if (hipEventSynchronize(r.end) != hipSuccess) return LRSA_ERR_HIP;
    if (hipEventElapsedTime(ms, r.beg, r.end) != hipSuccess) return LRSA_ERR_HIP;
    *name = r.name;
    return LRSA_OK;
}

}  // extern "C"
