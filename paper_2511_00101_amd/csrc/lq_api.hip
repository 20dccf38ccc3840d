// Entry points that launch nothing: status strings and the timing of the library's own launches.
#include <vector>

#include "lq_internal.h"

namespace lq {
namespace {
// (process-wide and not thread-safe, as the header says: benchmarks call this from one thread)
struct Record { int id; hipEvent_t e0, e1; };
bool g_profile = false;
std::vector<Record> g_records;
constexpr size_t kMaxRecords = 1 << 16;
void drop_records()
{
    for (const Record& r : g_records) {
        (void)hipEventDestroy(r.e0);
        (void)hipEventDestroy(r.e1);
    }
    g_records.clear();
}
}  // namespace

bool profile_on() { return g_profile; }

void profile_events(int kernel_id, hipEvent_t* start, hipEvent_t* stop)
{
    *start = *stop = nullptr;
    if (g_records.size() >= kMaxRecords) return;
    Record r{kernel_id, nullptr, nullptr};
    if (hipEventCreate(&r.e0) != hipSuccess) return;
    if (hipEventCreate(&r.e1) != hipSuccess) {
        (void)hipEventDestroy(r.e0);
        return;
    }
    g_records.push_back(r);
    *start = r.e0;
    *stop = r.e1;
}
}  // namespace lq

extern "C" lq_status lora_profile_enable(int32_t on)
{
    lq::drop_records();
    lq::g_profile = on != 0;
    return LQ_OK;
}

extern "C" lq_status lora_profile_read(double* total_us, int64_t* launches, int32_t n_kernels)
{
    if (!total_us || !launches || n_kernels < LQ_KERNEL_IDS) return LQ_ERR_INVALID_ARG;
    for (int i = 0; i < n_kernels; ++i) {
        total_us[i] = 0.0;
        launches[i] = 0;
    }
    lq_status status = LQ_OK;
    for (const lq::Record& r : lq::g_records) {
        float ms = 0.f;
        if (hipEventSynchronize(r.e1) != hipSuccess || hipEventElapsedTime(&ms, r.e0, r.e1) != hipSuccess) {
            status = LQ_ERR_HIP;
            continue;
        }
        total_us[r.id] += 1e3 * (double)ms;
        launches[r.id] += 1;
    }
    lq::drop_records();
    return status;
}

extern "C" size_t lora_workspace_bytes(int32_t n_tokens, int32_t n_adapters, int32_t max_rank, int32_t d_in, int32_t d_out)
{
    size_t need = lora_build_workspace_bytes(n_tokens, n_adapters);
    for (int variant = LQ_VARIANT_SPLIT; variant <= LQ_VARIANT_EXPAND_ONLY; ++variant) {
        const size_t f = lora_forward_workspace_bytes(n_tokens, max_rank, d_in, d_out, variant);
        if (f > need) need = f;
    }
    const size_t b = lora_backward_workspace_bytes(n_tokens, n_adapters, max_rank, d_in, d_out);
    return b > need ? b : need;
}

extern "C" const char* lora_status_string(lq_status status)
{
    switch (status) {
        case LQ_OK: return "ok";
        case LQ_ERR_INVALID_ARG: return "invalid argument";
        case LQ_ERR_UNSUPPORTED: return "unsupported shape, alignment, rank or adapter count";
        case LQ_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case LQ_ERR_HIP: return "HIP launch error";
    }
    return "unknown status";
}
