#include "ktimer.hpp"

#include <stdint.h>
#include <string.h>

#include <string>
#include <vector>

#include "../../include/hmmscan.h"

namespace hmm {
namespace {

struct Record { int name; hipEvent_t e0, e1; };
bool g_on = false;
std::vector<std::string> g_names;
std::vector<Record> g_records;
std::vector<hipEvent_t> g_pool;
size_t g_pool_used = 0;
struct Agg { double ms; int64_t n; };
std::vector<Agg> g_agg;
bool g_agg_valid = false;

hipEvent_t take_event() {
    if (g_pool_used == g_pool.size()) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        g_pool.push_back(e);
    }
    return g_pool[g_pool_used++];
}

int name_id(const char* name) {
    for (size_t i = 0; i < g_names.size(); ++i)
        if (g_names[i] == name) return (int)i;
    g_names.emplace_back(name);
    return (int)g_names.size() - 1;
}

void aggregate() {
    if (g_agg_valid) return;
    g_agg.assign(g_names.size(), Agg{0.0, 0});
    for (const Record& r : g_records) {
        if (!r.e0 || !r.e1) continue;
        if (hipEventSynchronize(r.e1) != hipSuccess) continue;
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, r.e0, r.e1) != hipSuccess) continue;
        g_agg[r.name].ms += ms;
        g_agg[r.name].n += 1;
    }
    g_agg_valid = true;
}

}  // namespace

bool ktimer_enabled() { return g_on; }

void ktimer_new_record(const char* name, hipEvent_t* start, hipEvent_t* stop) {
    Record r{name_id(name), take_event(), take_event()};
    g_records.push_back(r);
    g_agg_valid = false;
    *start = r.e0;
    *stop = r.e1;
}

}  // namespace hmm

extern "C" {

hmm_status hmm_kernel_timing_enable(int32_t on) {
    hmm::g_on = on != 0;
    hmm::g_records.clear();
    hmm::g_names.clear();
    hmm::g_pool_used = 0;
    hmm::g_agg_valid = false;
    return HMM_OK;
}

int32_t hmm_kernel_timing_count(void) {
    hmm::aggregate();
    return (int32_t)hmm::g_names.size();
}

hmm_status hmm_kernel_timing_get(int32_t index, const char** name, double* total_ms, int64_t* launches) {
    hmm::aggregate();
    if (index < 0 || index >= (int32_t)hmm::g_names.size() || !name || !total_ms || !launches)
        return HMM_ERR_INVALID_ARG;
    *name = hmm::g_names[index].c_str();
    *total_ms = hmm::g_agg[index].ms;
    *launches = hmm::g_agg[index].n;
    return HMM_OK;
}

}  // extern "C"
