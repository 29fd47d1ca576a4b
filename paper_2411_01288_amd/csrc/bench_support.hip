// Measurement support (declared in include/hexa_moe_bench.h; not part of the layer's interface):
// per-kernel timing of the library's own launches with HIP events on the launch stream.
// This is the only code in the library that creates HIP objects.
#include "common.h"
#include "../../include/hexa_moe_bench.h"

#include <cstring>
#include <mutex>
#include <vector>

namespace {

struct ProfRec { const char* label; hipEvent_t a, b; };
std::mutex g_mu;            // guards everything below
bool g_prof_on = false;
std::vector<ProfRec> g_prof;

}  // namespace

void prof_begin(hipStream_t st, const char* label) {
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_prof_on) return;
    ProfRec r{label, nullptr, nullptr};
    if (hipEventCreate(&r.a) != hipSuccess) return;
    if (hipEventCreate(&r.b) != hipSuccess) { (void)hipEventDestroy(r.a); return; }
    (void)hipEventRecord(r.a, st);
    g_prof.push_back(r);
}

// Closes the youngest record with this label that is still open (launch sequences of two host
// threads may interleave).
void prof_end(hipStream_t st, const char* label) {
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_prof_on) return;
    for (size_t i = g_prof.size(); i-- > 0;)
        if (g_prof[i].label == label) { (void)hipEventRecord(g_prof[i].b, st); return; }
}

extern "C" {

void hexa_moe_profile_enable(int on) {
    std::lock_guard<std::mutex> lk(g_mu);
    for (ProfRec& r : g_prof) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    g_prof.clear();
    g_prof_on = on != 0;
}

int hexa_moe_profile_read(int i, const char** label, float* ms_total, int* launches) {
    std::lock_guard<std::mutex> lk(g_mu);
    // distinct labels in first-seen order
    std::vector<const char*> names;
    for (const ProfRec& r : g_prof) {
        bool seen = false;
        for (const char* n : names) seen = seen || std::strcmp(n, r.label) == 0;
        if (!seen) names.push_back(r.label);
    }
    if (i < 0 || i >= (int)names.size()) return 0;
    float total = 0.f;
    int cnt = 0;
    for (const ProfRec& r : g_prof) {
        if (std::strcmp(r.label, names[i]) != 0) continue;
        float ms = 0.f;
        if (hipEventSynchronize(r.b) != hipSuccess) return 0;
        if (hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) return 0;
        total += ms;
        ++cnt;
    }
    *label = names[i]; *ms_total = total; *launches = cnt;
    return 1;
}

}  // extern "C"
