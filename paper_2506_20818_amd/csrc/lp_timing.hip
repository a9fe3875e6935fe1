// Optional instrumentation behind lp_timing_enable / lp_timing_collect: when switched on, every kernel launch of
// the library is bracketed by two HIP events recorded on the launch stream, and the elapsed times are summed per
// kernel class.  Off by default; the only process-global state of the library lives here.
#include "lp_internal.h"

#include <mutex>
#include <vector>

namespace {

struct Span {
    int cls;
    hipEvent_t beg, end;
};

std::mutex g_mu;
int g_level = 0;  // 0 off, 1 the main kernel classes, 2 every launch
std::vector<Span> g_spans;
std::vector<hipEvent_t> g_free;

hipEvent_t get_event() {
    if (!g_free.empty()) {
        hipEvent_t e = g_free.back();
        g_free.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

}  // namespace

LpTimedScope::LpTimedScope(int cls, hipStream_t st) : cls_(cls), st_(st), beg_(nullptr) {
    std::lock_guard<std::mutex> lock(g_mu);
    if (g_level == 0 || (g_level == 1 && cls_ == LP_KC_OTHER)) return;
    beg_ = get_event();
    if (beg_) (void)hipEventRecord(static_cast<hipEvent_t>(beg_), st_);
}

LpTimedScope::~LpTimedScope() {
    if (!beg_) return;
    std::lock_guard<std::mutex> lock(g_mu);
    hipEvent_t end = get_event();
    if (!end) {
        g_free.push_back(static_cast<hipEvent_t>(beg_));
        return;
    }
    (void)hipEventRecord(end, st_);
    g_spans.push_back(Span{cls_, static_cast<hipEvent_t>(beg_), end});
}

extern "C" int lp_timing_enable(int on) {
    std::lock_guard<std::mutex> lock(g_mu);
    g_level = on < 0 ? 0 : (on > 2 ? 2 : on);
    return LP_OK;
}

extern "C" int lp_timing_collect(double *ms_by_class, int64_t *launches_by_class, int32_t n_classes) {
    if (!ms_by_class || !launches_by_class || n_classes < LP_KC_COUNT) return LP_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_mu);
    for (int i = 0; i < n_classes; ++i) {
        ms_by_class[i] = 0.0;
        launches_by_class[i] = 0;
    }
    int status = LP_OK;
    for (const Span &s : g_spans) {
        float ms = 0.f;
        if (hipEventSynchronize(s.end) != hipSuccess || hipEventElapsedTime(&ms, s.beg, s.end) != hipSuccess) status = LP_ERR_HIP;
        ms_by_class[s.cls] += ms;
        launches_by_class[s.cls] += 1;
        g_free.push_back(s.beg);
        g_free.push_back(s.end);
    }
    g_spans.clear();
    return status;
}
