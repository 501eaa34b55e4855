// Environment switches of the library, read once per process (host code only).
#include "common.h"

#include <atomic>
#include <mutex>
#include <stdlib.h>
#include <string.h>

namespace ngc {

namespace {
const char *const kNames[SW_COUNT] = {"NGC_CONV3D_RANK2", "NGC_CONV3D_STRIP", "NGC_DB_FUSE", "NGC_G1_NCHW", "NGC_G1_VARIANT", "NGC_GEMM1X1", "NGC_STEM_BH", "NGC_STEM_TP", "NGC_STRIP_BW", "NGC_STRIP_MERGE", "NGC_STRIP_NF", "NGC_STRIP_ROWS", "NGC_STRIP_STRIDED", "NGC_STRIP_XCD", "NGC_WGG3_PARTS", "NGC_WGG_SLOTS", "NGC_WGG_SP", "NGC_WGG_TILE", "NGC_WGG_XCD", "NGC_WGRAD_G1", "NGC_WGRAD_GEMM", "NGC_WGRAD_LATE", "NGC_WGRAD_NCQ", "NGC_WGRAD_RING", "NGC_WGRAD_STRIP", "NGC_WSTEM_POS", "NGC_WSTEM_RING", "NGC_ROWS", "NGC_ROWS_LATE", "NGC_STAGED", "NGC_STRIP_TAIL", "NGC_STRIP_SPLIT", "NGC_WGRAD_NT", "NGC_STRIP_CPS", "NGC_DRY_RUN"};
char *g_val[SW_COUNT] = {};
std::atomic<uint32_t> g_epoch{0};
std::atomic<int> g_dry{0};
std::once_flag g_once;
std::mutex g_lock;

void load()
{
    std::lock_guard<std::mutex> g(g_lock);
    for (int i = 0; i < SW_COUNT; ++i) {
        const char *v = getenv(kNames[i]);
        // values handed out earlier stay valid: a changed value gets a new copy, the old one is kept
        if (v && g_val[i] && strcmp(v, g_val[i]) == 0) continue;
        g_val[i] = v ? strdup(v) : nullptr;
    }
    g_dry.store(g_val[SW_DRY_RUN] && atoi(g_val[SW_DRY_RUN]) == 1 ? 1 : 0);
}
}  // namespace

const char *env_switch(Switch s)
{
    std::call_once(g_once, load);
    return g_val[s];
}

uint32_t sw_epoch() { return g_epoch.load(std::memory_order_relaxed); }

bool dry_run()
{
    std::call_once(g_once, load);
    return g_dry.load(std::memory_order_relaxed) != 0;
}

}  // namespace ngc

extern "C" void ngc_reload_switches(void)
{
    std::call_once(ngc::g_once, ngc::load);
    ngc::load();
    ngc::g_epoch.fetch_add(1);
}
