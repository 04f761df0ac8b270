// Error state, version and small host utilities of libhyb.
#include "common.h"

#include <string.h>

#include <map>
#include <mutex>
#include <string>
#include <vector>

static thread_local char g_err[512] = "no error";

int hyb_set_error(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int hyb_check_launch(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hyb_set_error(HYB_ERR_LAUNCH, "%s: kernel launch failed: %s", what, hipGetErrorString(e));
    return HYB_OK;
}

extern "C" int hyb_version(void) { return 100; }

extern "C" const char* hyb_last_error_string(void) { return g_err; }

// ---- tracing -----------------------------------------------------------------------------------
namespace {
struct TraceRec { hipEvent_t e0, e1; int key; double work; };
struct TraceKey { std::string name, unit; };
std::mutex g_tmx;
bool g_trace_on = false;
std::vector<TraceRec> g_recs;          // records in use: [0, g_used)
size_t g_used = 0;
std::vector<TraceKey> g_keys;
std::map<std::string, int> g_key_index;
}  // namespace

HybTraceScope::HybTraceScope(const char* kernel, const char* unit, double work, hipStream_t stream) : slot(-1), st(stream) {
    if (!g_trace_on) return;
    std::lock_guard<std::mutex> lk(g_tmx);
    auto it = g_key_index.find(kernel);
    int key;
    if (it == g_key_index.end()) {
        key = (int)g_keys.size();
        g_keys.push_back({kernel, unit});
        g_key_index[kernel] = key;
    } else {
        key = it->second;
    }
    if (g_used == g_recs.size()) {
        TraceRec r;
        if (hipEventCreate(&r.e0) != hipSuccess || hipEventCreate(&r.e1) != hipSuccess) return;
        g_recs.push_back(r);
    }
    slot = (int)g_used++;
    g_recs[slot].key = key;
    g_recs[slot].work = work;
    (void)hipEventRecord(g_recs[slot].e0, st);
}

HybTraceScope::~HybTraceScope() {
    if (slot < 0) return;
    std::lock_guard<std::mutex> lk(g_tmx);
    (void)hipEventRecord(g_recs[slot].e1, st);
}

extern "C" int hyb_trace_enable(int on) {
    std::lock_guard<std::mutex> lk(g_tmx);
    g_trace_on = on != 0;
    if (g_trace_on) g_used = 0;
    return HYB_OK;
}

extern "C" int hyb_trace_summary(char* buf, size_t cap) {
    HYB_REQUIRE(buf != nullptr && cap > 0, HYB_ERR_NULL, "hyb_trace_summary: no buffer");
    std::lock_guard<std::mutex> lk(g_tmx);
    struct Acc { double ms = 0, work = 0; long count = 0; };
    std::vector<Acc> acc(g_keys.size());
    for (size_t i = 0; i < g_used; i++) {
        float ms = 0.f;
        if (hipEventSynchronize(g_recs[i].e1) != hipSuccess || hipEventElapsedTime(&ms, g_recs[i].e0, g_recs[i].e1) != hipSuccess)
            return hyb_set_error(HYB_ERR_LAUNCH, "hyb_trace_summary: event query failed");
        Acc& a = acc[g_recs[i].key];
        a.ms += ms; a.work += g_recs[i].work; a.count++;
    }
    size_t off = 0;
    buf[0] = 0;
    for (size_t k = 0; k < g_keys.size(); k++) {
        if (!acc[k].count) continue;
        int w = snprintf(buf + off, cap - off, "%s\t%s\t%ld\t%.6f\t%.6e\n", g_keys[k].name.c_str(), g_keys[k].unit.c_str(),
                         acc[k].count, acc[k].ms, acc[k].work);
        if (w < 0 || (size_t)w >= cap - off) return hyb_set_error(HYB_ERR_WORKSPACE, "hyb_trace_summary: buffer of %zu bytes is too small", cap);
        off += (size_t)w;
    }
    return HYB_OK;
}
