// Per-launch timing facility behind fhpc_profile_*: a fixed pool of event pairs that
// the launch wrappers record around each kernel while profiling is switched on.
#include "../../include/fingpt_hpc.h"
#include "profile.h"

#include <string.h>
#include <vector>

namespace fhpc {

namespace {
struct Record {
    hipEvent_t start, stop;
    char name[64];
    double flops, bytes;
};
std::vector<Record> g_pool;
int g_count = 0;
bool g_on = false;
}  // namespace

bool prof_on() { return g_on; }

int prof_begin(const char* name, double flops, double bytes, hipStream_t s)
{
    if (!g_on || g_count >= (int)g_pool.size()) return -1;
    Record& r = g_pool[g_count];
    strncpy(r.name, name, sizeof(r.name) - 1);
    r.name[sizeof(r.name) - 1] = 0;
    r.flops = flops;
    r.bytes = bytes;
    if (hipEventRecord(r.start, s) != hipSuccess) return -1;
    return g_count++;
}

void prof_end(int slot, hipStream_t s)
{
    if (slot >= 0) (void)hipEventRecord(g_pool[slot].stop, s);
}

}  // namespace fhpc

using namespace fhpc;

extern "C" {

int fhpc_profile_start(int max_records)
{
    if (max_records < 1) return FHPC_ERR_SHAPE;
    while ((int)g_pool.size() < max_records) {
        Record r;
        memset(&r, 0, sizeof(r));
        if (hipEventCreate(&r.start) != hipSuccess || hipEventCreate(&r.stop) != hipSuccess) return FHPC_ERR_HIP;
        g_pool.push_back(r);
    }
    g_count = 0;
    g_on = true;
    return FHPC_OK;
}

int fhpc_profile_stop(void)
{
    g_on = false;
    return g_count;
}

int fhpc_profile_get(int index, char* name, int name_len, float* ms, double* flops, double* bytes)
{
    if (index < 0 || index >= g_count || !name || name_len < 1 || !ms || !flops || !bytes) return FHPC_ERR_SHAPE;
    Record& r = g_pool[index];
    if (hipEventSynchronize(r.stop) != hipSuccess) return FHPC_ERR_HIP;
    if (hipEventElapsedTime(ms, r.start, r.stop) != hipSuccess) return FHPC_ERR_HIP;
    strncpy(name, r.name, (size_t)name_len - 1);
    name[name_len - 1] = 0;
    *flops = r.flops;
    *bytes = r.bytes;
    return FHPC_OK;
}

}  // extern "C"
