// Event pool behind the optional per-kernel timing.
#include "profile.h"
#include "../../include/gswa.h"

#include <mutex>
#include <vector>

namespace gswa {

namespace {
struct Slot {
    hipEvent_t start, stop;
    int id;
};
std::mutex g_mu;
std::vector<Slot> g_pool;
size_t g_used = 0;
long long g_dropped = 0;
bool g_on = false;
constexpr size_t kPool = 8192;
} // namespace

const char *kernel_name(int id)
{
    static const char *names[K_COUNT] = {"fill_zero", "qkv_linear", "attn_fwd", "proj_linear",
                                         "proj_wgrad", "dO_linear", "attn_bwd", "dx_linear",
                                         "qkv_wgrad", "pack_fwd", "fused_fwd", "fused_bwd", "reduce_partials", "fused_attn_fwd", "proj_gemm",
                                         "wproj_grad", "attn_core_fwd", "attn_core_bwd", "qkv+dO_linear", "window_fwd",
                                         "ln_fwd", "ln_bwd", "gelu_fwd", "gelu_bwd", "fc1_linear", "fc2_linear",
                                         "fc_dlinear", "fc_wgrad", "mlp_fwd", "mlp_bwd", "mlp_pack", "mlp_reduce", "ln_fwd+mlp_reduce",
                                         "wide_attn_bwd", "wide_qkv_grad"};
    return (id >= 0 && id < K_COUNT) ? names[id] : "?";
}

KernelTimer::KernelTimer(int id, hipStream_t s) : slot(-1), stream(s)
{
    if (!g_on) return;
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_on) return;
    if (g_used >= g_pool.size()) {
        ++g_dropped;
        return;
    }
    slot = (int)g_used++;
    g_pool[slot].id = id;
    (void)hipEventRecord(g_pool[slot].start, stream);
}

KernelTimer::~KernelTimer()
{
    if (slot >= 0) (void)hipEventRecord(g_pool[slot].stop, stream);
}

} // namespace gswa

extern "C" {

int gswa_profile_enable(int on)
{
    using namespace gswa;
    std::lock_guard<std::mutex> lk(g_mu);
    if (on && g_pool.empty()) {
        g_pool.resize(kPool);
        for (auto &s : g_pool) {
            if (hipEventCreate(&s.start) != hipSuccess || hipEventCreate(&s.stop) != hipSuccess) {
                g_pool.clear();
                return GSWA_EHIP;
            }
        }
    }
    g_on = on != 0;
    return GSWA_OK;
}

int gswa_profile_kernel_count(void) { return gswa::K_COUNT; }

const char *gswa_profile_kernel_name(int id) { return gswa::kernel_name(id); }

int gswa_profile_collect(double *total_ms, long long *launches, long long *dropped)
{
    using namespace gswa;
    std::lock_guard<std::mutex> lk(g_mu);
    for (int i = 0; i < K_COUNT; ++i) {
        if (total_ms) total_ms[i] = 0.0;
        if (launches) launches[i] = 0;
    }
    int rc = GSWA_OK;
    for (size_t i = 0; i < g_used; ++i) {
        float ms = 0.f;
        if (hipEventSynchronize(g_pool[i].stop) != hipSuccess ||
            hipEventElapsedTime(&ms, g_pool[i].start, g_pool[i].stop) != hipSuccess) {
            rc = GSWA_EHIP;
            continue;
        }
        if (total_ms) total_ms[g_pool[i].id] += ms;
        if (launches) launches[g_pool[i].id] += 1;
    }
    if (dropped) *dropped = g_dropped;
    g_used = 0;
    g_dropped = 0;
    return rc;
}

} // extern "C"
