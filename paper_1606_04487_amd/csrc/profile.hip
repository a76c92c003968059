// Optional per-kernel timing with HIP events on the caller's stream.
//
// When switched on, every kernel launch of the library is bracketed by two events recorded on the
// stream the kernel runs on, together with the algorithmic work of that launch (flops for the
// GEMMs, bytes for the data-movement kernels).  omni_profile_summary() waits for the events and
// adds up the elapsed times per kernel class.  Off by default: the launch path then costs one
// branch.  Events are created on demand and reused; this is the only place the library creates
// HIP objects, and only while profiling is on.
#include <mutex>
#include <vector>

#include "common.h"

namespace omni {

static const char *const kNames[KID_COUNT] = {
    "lower", "pack_khat", "pack_dyhat", "bias_reduce", "gemm_forward", "gemm_dgrad", "gemm_wgrad",
    "reduce_partials", "col2im", "sgd", "relu", "maxpool_forward", "maxpool_backward", "conv_fused_forward", "conv_fused_dgrad", "conv_strided_forward",
    "lrn", "dropout",
};

struct Record { int kid; hipEvent_t start, stop; double flops, bytes; };

static std::mutex g_mu;
static bool g_on = false;
static uint64_t g_mask = ~0ull;  // kernel classes that are recorded (bit k = class k)
static std::vector<Record> g_records;
static std::vector<hipEvent_t> g_free;
static const size_t kMaxRecords = 1u << 20;
static_assert(KID_COUNT <= 64, "kernel classes fit the selection mask");

bool profile_enabled() { return g_on; }

static hipEvent_t get_event()
{
    if (!g_free.empty()) {
        hipEvent_t e = g_free.back();
        g_free.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

ProfScope::ProfScope(int kid, hipStream_t s, double flops, double bytes) : slot_(-1), stream_(s)
{
    if (!g_on || !((g_mask >> kid) & 1ull)) return;
    std::lock_guard<std::mutex> lock(g_mu);
    if (g_records.size() >= kMaxRecords) return;
    Record r{kid, get_event(), get_event(), flops, bytes};
    if (r.start == nullptr || r.stop == nullptr) return;
    (void)hipEventRecord(r.start, s);
    g_records.push_back(r);
    slot_ = (long)g_records.size() - 1;
}

ProfScope::~ProfScope()
{
    if (slot_ < 0) return;
    std::lock_guard<std::mutex> lock(g_mu);
    if ((size_t)slot_ < g_records.size()) (void)hipEventRecord(g_records[slot_].stop, stream_);
}

}  // namespace omni

using namespace omni;

extern "C" {

int omni_profile_enable(int on)
{
    std::lock_guard<std::mutex> lock(g_mu);
    for (Record &r : g_records) {
        g_free.push_back(r.start);
        g_free.push_back(r.stop);
    }
    g_records.clear();
    g_on = on != 0;
    g_mask = ~0ull;
    return OMNI_OK;
}

int omni_profile_select(int kernel_id)
{
    if (kernel_id < -1 || kernel_id >= KID_COUNT) return OMNI_INVALID_ARGUMENT;
    std::lock_guard<std::mutex> lock(g_mu);
    g_mask = kernel_id < 0 ? ~0ull : (1ull << kernel_id);
    return OMNI_OK;
}

int omni_profile_select_mask(uint64_t mask)
{
    std::lock_guard<std::mutex> lock(g_mu);
    g_mask = mask;
    return OMNI_OK;
}

int omni_profile_kernel_count(void) { return KID_COUNT; }

const char *omni_profile_kernel_name(int kernel_id)
{
    return (kernel_id >= 0 && kernel_id < KID_COUNT) ? kNames[kernel_id] : "";
}

int omni_profile_summary(int kernel_id, int64_t *launches, double *total_ms, double *flops, double *bytes)
{
    if (kernel_id < 0 || kernel_id >= KID_COUNT || !launches || !total_ms || !flops || !bytes)
        return OMNI_INVALID_ARGUMENT;
    std::lock_guard<std::mutex> lock(g_mu);
    *launches = 0;
    *total_ms = *flops = *bytes = 0.0;
    for (const Record &r : g_records) {
        if (r.kid != kernel_id) continue;
        if (hipEventSynchronize(r.stop) != hipSuccess) return OMNI_HIP_ERROR;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) return OMNI_HIP_ERROR;
        *launches += 1;
        *total_ms += ms;
        *flops += r.flops;
        *bytes += r.bytes;
    }
    return OMNI_OK;
}

}  // extern "C"
