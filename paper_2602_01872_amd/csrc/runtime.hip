// Error reporting and per-kernel event timing for libgrappa_hip.so.
#include "common.h"

#include <map>
#include <mutex>
#include <vector>

namespace grp {

static thread_local std::string g_err;

void set_error(const char* fmt, ...) {
    char buf[1024];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
}

grp_status fail(grp_status code, const char* fmt, ...) {
    char buf[1024];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

struct ProfRec {
    std::string name;
    hipEvent_t a, b;
    double flops, bytes;
};
static std::mutex g_prof_mu;
static bool g_prof_on = false;
static std::vector<ProfRec> g_prof;
static thread_local hipEvent_t g_open_end = nullptr;
static bool g_prof_detail = false;           // enable value 2: kernel names carry the launch shape
static thread_local char g_detail[96] = {0};

void prof_detail(const char* fmt, ...) {
    if (!g_prof_on || !g_prof_detail) return;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_detail, sizeof g_detail, fmt, ap);
    va_end(ap);
}

void prof_begin(const char* name, hipStream_t st, double flops, double bytes) {
    if (!g_prof_on) return;
    ProfRec r{name, nullptr, nullptr, flops, bytes};
    if (g_prof_detail && g_detail[0]) { r.name += g_detail; }
    g_detail[0] = 0;
    if (hipEventCreate(&r.a) != hipSuccess || hipEventCreate(&r.b) != hipSuccess) return;
    (void)hipEventRecord(r.a, st);
    g_open_end = r.b;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    g_prof.push_back(r);
}

void prof_end(hipStream_t st) {
    if (!g_prof_on || !g_open_end) return;
    (void)hipEventRecord(g_open_end, st);
    g_open_end = nullptr;
}

// One helper stream (default priority, not synchronising with the legacy stream) and its events per caller
// stream and device, created at the first request and kept until the process ends.
SideLane* side_lane(hipStream_t main) {
    static std::mutex mu;
    static std::map<std::pair<int, hipStream_t>, SideLane*> lanes;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
    std::lock_guard<std::mutex> lk(mu);
    auto it = lanes.find({dev, main});
    if (it != lanes.end()) return it->second;
    if (main) {            // nothing is created while the caller's stream is being captured
        hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(main, &cs) != hipSuccess || cs != hipStreamCaptureStatusNone) {
            (void)hipGetLastError();
            return nullptr;
        }
    }
    SideLane* lane = new SideLane();
    bool ok = hipStreamCreateWithFlags(&lane->stream, hipStreamNonBlocking) == hipSuccess;
    for (int l = 0; ok && l < GRP_MAX_LAYERS; ++l)
        ok = hipEventCreateWithFlags(&lane->fork[l], hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&lane->join, hipEventDisableTiming) == hipSuccess;
    if (!ok) {             // the step then runs on the caller's stream alone; what was created stays allocated
        (void)hipGetLastError();
        return nullptr;
    }
    lanes[{dev, main}] = lane;
    return lane;
}

}  // namespace grp

extern "C" const char* grp_last_error(void) { return grp::g_err.c_str(); }

extern "C" grp_status grp_profile_enable(int32_t on) {
    std::lock_guard<std::mutex> lk(grp::g_prof_mu);
    grp::g_prof_on = on != 0;
    grp::g_prof_detail = on == 2;
    return GRP_OK;
}

extern "C" grp_status grp_profile_report(char* buf, size_t cap) {
    if (!buf || cap == 0) return grp::fail(GRP_EINVAL, "grp_profile_report: null buffer");
    std::vector<grp::ProfRec> recs;
    {
        std::lock_guard<std::mutex> lk(grp::g_prof_mu);
        recs.swap(grp::g_prof);
    }
    struct Acc { long n; double ms, flops, bytes; };
    std::map<std::string, Acc> acc;
    std::vector<std::string> order;
    for (auto& r : recs) {
        float ms = 0.f;
        if (hipEventSynchronize(r.b) == hipSuccess && hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) {
            auto it = acc.find(r.name);
            if (it == acc.end()) {
                order.push_back(r.name);
                acc[r.name] = Acc{1, ms, r.flops, r.bytes};
            } else {
                it->second.n += 1;
                it->second.ms += ms;
                it->second.flops += r.flops;
                it->second.bytes += r.bytes;
            }
        }
        (void)hipEventDestroy(r.a);
        (void)hipEventDestroy(r.b);
    }
    std::string out;
    char line[320];
    for (auto& nm : order) {
        const Acc& a = acc[nm];
        snprintf(line, sizeof line, "%s %ld %.6f %.6e %.6e\n", nm.c_str(), a.n, a.ms, a.flops, a.bytes);
        out += line;
    }
    if (out.size() + 1 > cap) out.resize(cap - 1);
    memcpy(buf, out.c_str(), out.size() + 1);
    return GRP_OK;
}
