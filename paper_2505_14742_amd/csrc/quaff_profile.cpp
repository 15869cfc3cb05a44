// Optional per-launch timing of the library's kernels with HIP events on the caller's stream.
// Off by default; when off the launchers pay one relaxed atomic load.
#include <atomic>
#include <mutex>
#include <vector>

#include "../../include/quaff.h"
#include "quaff_internal.h"

namespace quaff {

namespace {
struct Rec {
    int kind;
    hipEvent_t start, stop;
};
std::atomic<int> g_on{0};
std::mutex g_mu;
std::vector<Rec> g_recs;
std::vector<float> g_ms;           // filled by collect()
constexpr size_t kMaxRecs = 1 << 16;
const char* kNames[KERNEL_KINDS] = {"prepare_weight", "colmax_outlier", "momentum_what", "quant_rows", "lora_down",
                                    "gemm_i8", "lora_grad", "outlier_grad", "calibrate", "quant_rows+lora_down", "colmax_outlier+lora_down",
                                    "momentum_what+quant_rows", "fwd_prep"};
}  // namespace

ProfScope::ProfScope(int kind, hipStream_t stream) : stream_(stream), idx_(-1) {
    if (!g_on.load(std::memory_order_relaxed)) return;
    std::lock_guard<std::mutex> lk(g_mu);
    if (g_recs.size() >= kMaxRecs) return;
    Rec r{kind, nullptr, nullptr};
    if (hipEventCreate(&r.start) != hipSuccess) return;
    if (hipEventCreate(&r.stop) != hipSuccess) { (void)hipEventDestroy(r.start); return; }
    (void)hipEventRecord(r.start, stream);
    g_recs.push_back(r);
    idx_ = (int)g_recs.size() - 1;
}

ProfScope::~ProfScope() {
    if (idx_ < 0) return;
    std::lock_guard<std::mutex> lk(g_mu);
    (void)hipEventRecord(g_recs[idx_].stop, stream_);
}

}  // namespace quaff

extern "C" {

int quaff_profile_enable(int on) {
    using namespace quaff;
    std::lock_guard<std::mutex> lk(g_mu);
    for (auto& r : g_recs) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
    g_recs.clear();
    g_ms.clear();
    g_on.store(on ? 1 : 0);
    return QUAFF_OK;
}

int64_t quaff_profile_collect(void) {
    using namespace quaff;
    std::lock_guard<std::mutex> lk(g_mu);
    g_ms.assign(g_recs.size(), 0.0f);
    for (size_t i = 0; i < g_recs.size(); ++i) {
        if (hipEventSynchronize(g_recs[i].stop) != hipSuccess) return -1;
        if (hipEventElapsedTime(&g_ms[i], g_recs[i].start, g_recs[i].stop) != hipSuccess) return -1;
    }
    return (int64_t)g_recs.size();
}

int quaff_profile_launch(int64_t index, int* kind, float* ms) {
    using namespace quaff;
    std::lock_guard<std::mutex> lk(g_mu);
    if (index < 0 || (size_t)index >= g_ms.size() || !kind || !ms) return QUAFF_ERR_SHAPE;
    *kind = g_recs[index].kind;
    *ms = g_ms[index];
    return QUAFF_OK;
}

const char* quaff_profile_kind_name(int kind) {
    return (kind >= 0 && kind < quaff::KERNEL_KINDS) ? quaff::kNames[kind] : "unknown";
}

}  // extern "C"
