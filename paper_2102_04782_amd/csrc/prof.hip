// Measurement aid: optional HIP-event bracketing of every kernel launch of the library.
#include <string.h>

#include <atomic>
#include <mutex>
#include <string>
#include <vector>

#include "daq_internal.h"

namespace daq {

namespace {
struct Span {
    std::string name;
    hipEvent_t start, stop;
};
std::atomic<bool> g_active{false};
std::mutex g_mu;            // guards everything below
bool g_calibrated = false;
std::vector<Span> g_spans;
}  // namespace

bool prof_active() { return g_active.load(std::memory_order_relaxed); }

void prof_push(const char* name, hipStream_t s) {
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_calibrated) {
        // An event pair with nothing between it measures what the bracketing itself adds to every span.
        g_calibrated = true;
        for (int i = 0; i < 8; ++i) {
            Span c;
            c.name = "(empty event pair)";
            if (hipEventCreate(&c.start) != hipSuccess || hipEventCreate(&c.stop) != hipSuccess) break;
            (void)hipEventRecord(c.start, s);
            (void)hipEventRecord(c.stop, s);
            g_spans.push_back(c);
        }
    }
    Span sp;
    sp.name = name;
    if (hipEventCreate(&sp.start) != hipSuccess || hipEventCreate(&sp.stop) != hipSuccess) return;
    (void)hipEventRecord(sp.start, s);
    g_spans.push_back(sp);
}

void prof_pop(hipStream_t s) {
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_spans.empty()) (void)hipEventRecord(g_spans.back().stop, s);
}

}  // namespace daq

extern "C" {

daq_status daq_prof_begin(void) {
    std::lock_guard<std::mutex> lock(daq::g_mu);
    for (auto& sp : daq::g_spans) {
        (void)hipEventDestroy(sp.start);
        (void)hipEventDestroy(sp.stop);
    }
    daq::g_spans.clear();
    daq::g_active = true;
    daq::g_calibrated = false;
    return DAQ_OK;
}

daq_status daq_prof_end(daq_prof_row* rows, int32_t max_rows, int32_t* n_rows) {
    daq::g_active = false;
    std::lock_guard<std::mutex> lock(daq::g_mu);
    if (!rows || !n_rows || max_rows <= 0) return DAQ_ERR_INVALID_ARG;
    int n = 0;
    daq_status rc = DAQ_OK;
    for (auto& sp : daq::g_spans) {
        float ms = 0.f;
        if (hipEventSynchronize(sp.stop) != hipSuccess || hipEventElapsedTime(&ms, sp.start, sp.stop) != hipSuccess) {
            rc = DAQ_ERR_HIP;
            ms = 0.f;
        }
        int j = 0;
        for (; j < n; ++j)
            if (sp.name == rows[j].name) break;
        if (j == n) {
            if (n == max_rows) continue;
            memset(&rows[n], 0, sizeof(rows[n]));
            strncpy(rows[n].name, sp.name.c_str(), sizeof(rows[n].name) - 1);
            ++n;
        }
        rows[j].total_ms += ms;
        rows[j].launches += 1;
        (void)hipEventDestroy(sp.start);
        (void)hipEventDestroy(sp.stop);
    }
    daq::g_spans.clear();
    *n_rows = n;
    return rc;
}

}  // extern "C"
