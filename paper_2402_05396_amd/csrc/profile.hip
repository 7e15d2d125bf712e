// Optional per-kernel timing: between taser_profile_begin() and
// taser_profile_end() every kernel the library launches is bracketed by a pair
// of HIP events recorded on the stream it is launched on.
#include <cstring>
#include <string>
#include <vector>

#include "taser_internal.h"
#include "taser_profile.h"

namespace {

struct Span {
    hipEvent_t start, stop;
    const char* name;
};

bool g_enabled = false;
std::string g_only;               // non-empty: time only the kernel of this name
std::vector<Span> g_spans;        // spans of the current session
std::vector<hipEvent_t> g_pool;   // events free for reuse
constexpr size_t kMaxSpans = 1u << 16;

hipEvent_t take_event() {
    if (!g_pool.empty()) {
        hipEvent_t e = g_pool.back();
        g_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

}  // namespace

TaserProfileSpan::TaserProfileSpan(hipStream_t stream, const char* name) : stream_(stream), index_(-1) {
    if (!g_enabled || g_spans.size() >= kMaxSpans) return;
    if (!g_only.empty() && g_only != name) return;
    Span s{take_event(), take_event(), name};
    if (!s.start || !s.stop) return;
    if (hipEventRecord(s.start, stream) != hipSuccess) return;
    index_ = (long)g_spans.size();
    g_spans.push_back(s);
}

TaserProfileSpan::~TaserProfileSpan() {
    if (index_ >= 0) (void)hipEventRecord(g_spans[(size_t)index_].stop, stream_);
}

extern "C" int taser_profile_begin_only(const char* kernel_name) {
    const int rc = taser_profile_begin();
    g_only = kernel_name ? kernel_name : "";
    return rc;
}

extern "C" int taser_profile_begin(void) {
    g_only.clear();
    for (const Span& s : g_spans) {
        g_pool.push_back(s.start);
        g_pool.push_back(s.stop);
    }
    g_spans.clear();
    g_enabled = true;
    return TASER_OK;
}

extern "C" int taser_profile_end(taser_kernel_time* out, int32_t max_entries, int32_t* num_entries) {
    g_enabled = false;
    if (!num_entries || (max_entries > 0 && !out) || max_entries < 0)
        return taser_fail(TASER_E_ARG, "profile_end: bad output arguments");
    int32_t count = 0;
    int rc = TASER_OK;
    for (const Span& s : g_spans) {
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(s.stop);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, s.start, s.stop);
        if (e != hipSuccess) {
            rc = taser_fail_hip(e, "profile_end: reading an event pair");
            continue;
        }
        int32_t at = 0;
        while (at < count && std::strcmp(out[at].name, s.name) != 0) ++at;
        if (at == count) {
            if (count == max_entries) continue;   // table full: this kernel is not reported
            out[at].name = s.name;
            out[at].launches = 0;
            out[at].total_ms = 0.0;
            ++count;
        }
        out[at].launches += 1;
        out[at].total_ms += (double)ms;
    }
    for (const Span& s : g_spans) {
        g_pool.push_back(s.start);
        g_pool.push_back(s.stop);
    }
    g_spans.clear();
    *num_entries = count;
    return rc;
}
